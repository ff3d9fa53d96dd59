// On-chip path: one workgroup evaluates one whole snapshot (up to 8192 queued requests)
// with a single read of the inputs and a single write of the outputs.
//
// Per snapshot (paper Section 3.2 Eq.(1),(2),(4), DAG maximum; Section 3.3 ordering):
//   1. load deadline/stage (arrival for FCFS stages), form the order key
//   2. bucket every request by (stage, leading bits of key.index) with LDS counters;
//      the bucket order is the queue order, so an exclusive scan of the counters gives
//      every bucket's first queue slot and every stage's queue start and length
//   3. scatter the remaining low bits of key.index into LDS by bucket; a request's exact
//      rank is its bucket start plus the number of bucket mates with smaller low bits
//   4. per stage: cost at full queue length; per path entry: downstream suffix sum,
//      maximum per stage (the path CSR is walked here)
//   5. per request: own-stage cost at its queue position + downstream maximum,
//      drop decision; outputs leave in request order, the queue order via LDS.
//      Sequentially consistent variant: the position counts only the requests ahead that
//      were kept (the Request Broker takes a queue in order and a dropped request never
//      takes a batch slot, Section 4.1), so a queue is a chain of decisions; one wave walks
//      it 64 requests at a time and settles each group by iterating to the fixed point.
//
// Why buckets instead of radix passes: at this data rate the vector ALU, not HBM, limits a
// sort of 8192 keys per workgroup (about 130 lane-instructions per request at full HBM
// speed).  A stable 8-bit radix pass costs ~70 of them per key per pass.  One bucketing
// pass with ~0.7 requests per bucket and a compare loop over bucket mates costs less than
// one radix pass.  Appending the request index below the key makes equal keys spread over
// buckets too, so heavy ties stay cheap; only a strongly clustered key distribution
// degrades to many compares per request (still exact).
#include "pard_device.hpp"

namespace pard {

namespace {

// Capacity CAP (a power of two from 256 to PARD_FUSED_SNAPSHOT_CAPACITY) with CAP / 16 threads (more at 256, 512
// and 1024, where that measured faster or is what one wave needs): a
// workgroup sized for 8192 requests spends most of its time on fixed costs when a snapshot holds a
// few hundred, so smaller snapshots get smaller workgroups (and more of them per compute unit).
//
// SCAP is the number of stages the per-stage arrays and the latency-table cache are sized for.  Sized
// for PARD_MAX_STAGES they cost about 24 KB per workgroup, more than everything else a small
// capacity needs, and that alone would hold a compute unit to a few one-wave workgroups; pipelines
// of at most kFewStages stages (the usual case) therefore get a variant that carries a tenth of that, and
// those of at most kSomeStages one that carries a fifth (12 stages on 65,536 snapshots of 256: 0.41 ms with
// the full-size arrays).
constexpr int kFewStages = 8;
constexpr int kSomeStages = 16;

template <int CAP, int SCAP>
struct SnapshotLds {
    // 1.5 * CAP 16-bit counters, two per LDS word (2 * CAP at the smallest capacity: a thread scans an even number of words)
    static constexpr int kCntWords = CAP == 256 ? CAP : CAP * 3 / 4;
    static constexpr int kAuxMin = SCAP * PARD_LAT_ENTRIES + 256;   // words: every stage's latency table + path entries
    static constexpr int kAuxWords = CAP / 2 > kAuxMin ? CAP / 2 : kAuxMin;
    __align__(16) uint32_t cnt32[kCntWords + 4];     // bucket counters, then bucket starts; later the queue order
    __align__(16) uint32_t low[CAP + 4];             // per queue slot: low bits of key.index (or the whole key)
    __align__(16) uint16_t idx[2 * kAuxWords];       // per queue slot: local index (wide keys only); otherwise
                                                     // a cache: latency tables, then path entries
    StageRec recs[SCAP];
    unsigned long long cfull[SCAP];
    unsigned long long down[SCAP];
    int32_t seg_start[SCAP + 1];
    __align__(16) uint32_t quick[SCAP][8];   // per stage: B-1, 1/B, 1/W, aW, bW, queue start (short-queue form)
    uint32_t slow_stages;                            // set when some stage cannot use the short-queue form
    uint32_t wave_tot[16];
    uint32_t kept_tot[16][2];                        // survivor staging: kept slots per wave and group of loads
    uint32_t red[2];
};

constexpr int log2_of(int x) { return x <= 1 ? 0 : 1 + log2_of(x / 2); }

// FULL: the snapshot holds exactly kCap requests and every array is 16-byte aligned at its
// start, so no per-request bounds test is needed.
// Minimum over the lanes below (INT32_MAX in lane 0), on the vector ALU's data-parallel primitives.
__device__ __forceinline__ int32_t wave_exclusive_min(int32_t v) {
    const int32_t inf = kInt32Max;
    int32_t x = __builtin_amdgcn_update_dpp(inf, v, 0x138, 0xF, 0xF, false);          // wave_shr:1: the lane below's value
    auto lower = [](int32_t a, int32_t b) { return a < b ? a : b; };
    x = lower(x, __builtin_amdgcn_update_dpp(inf, x, 0x111, 0xF, 0xF, false));         // row_shr:1
    x = lower(x, __builtin_amdgcn_update_dpp(inf, x, 0x112, 0xF, 0xF, false));         // row_shr:2
    x = lower(x, __builtin_amdgcn_update_dpp(inf, x, 0x114, 0xF, 0xF, false));         // row_shr:4
    x = lower(x, __builtin_amdgcn_update_dpp(inf, x, 0x118, 0xF, 0xF, false));         // row_shr:8
    x = lower(x, __builtin_amdgcn_update_dpp(inf, x, 0x142, 0xA, 0xF, false));         // row_bcast:15 into rows 1, 3
    x = lower(x, __builtin_amdgcn_update_dpp(inf, x, 0x143, 0xC, 0xF, false));         // row_bcast:31 into rows 2, 3
    return x;
}

template <int T, int CAP, int SCAP, bool FULL, bool CONSISTENT>
__device__ __forceinline__ void snapshot_body(const FusedArgs& A, SnapshotLds<CAP, SCAP>& L, const int u, const int64_t lo,
                                              const int m, const bool aligned, const int off) {
    constexpr int kCap = CAP;
    constexpr int kIdxBits = log2_of(CAP);                 // bits of a local index
    constexpr int kCntWords = SnapshotLds<CAP, SCAP>::kCntWords;
    constexpr int kBuckets = 2 * kCntWords;                // 16-bit counters
    constexpr int kAuxWords = SnapshotLds<CAP, SCAP>::kAuxWords;
    constexpr int G = kCap / (4 * T);       // groups of 4 consecutive requests per thread
    constexpr int CW = kCntWords / T;       // counter words scanned per thread
    static_assert(kCap == (1 << kIdxBits) && kCap <= PARD_FUSED_SNAPSHOT_CAPACITY, "capacity");
    static_assert(G >= 1 && CW >= 2 && CW % 2 == 0 && kCntWords % T == 0 && T % kWave == 0 && T / kWave <= 16, "shape");

    const PlanDev& P = A.plan;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int S = P.S;
    const int dag = P.shared ? 0 : u;
    const int32_t* lat_dag = P.lat + (int64_t)dag * S * PARD_LAT_ENTRIES;
    // Local indices: request lo + i has local index i + off, where off = lo mod 4 when the arrays allow
    // 16-byte accesses (0 otherwise).  A thread's groups of four then sit on 16-byte boundaries of the
    // request arrays whatever the snapshot's first request is; the `off` slots before the snapshot
    // and the ones behind its end are simply not live.
    const int64_t lo_s = lo - off;
    const int m_s = m + off;
    auto live = [&](int idx) { return FULL || (idx >= off && idx < m_s); };
    auto whole = [&](int base) { return FULL || (aligned && base >= off && base + 3 < m_s); };   // four live requests, 16-byte access
    // a thread's g-th group of four lies in slots [g * 4T, (g + 1) * 4T): a snapshot that ends before them leaves
    // the whole workgroup nothing to do for that g, in any phase
    auto dead_group = [&](int g) { return !FULL && g * T * 4 >= m_s; };
    uint32_t* aux = reinterpret_cast<uint32_t*>(L.idx);           // kAuxWords words
    const int e_lo = P.dag_entry_ptr[dag], n_entries = P.dag_entry_ptr[dag + 1] - e_lo;
    const bool entries_cached = S * PARD_LAT_ENTRIES + n_entries <= kAuxWords;
    const int32_t now = A.now[u];

    // ---- 1. loads (issued first), LDS initialisation meanwhile ---------------
    int32_t dl[G][4], st[G][4];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        if (dead_group(g)) continue;
        const int base = (g * T + tid) * 4;
        if (FULL || (aligned && base < m_s && lo_s + base + 3 < A.n)) {      // neighbours' values may ride along: they are not live
            // read once: streaming loads (measured with the request order shuffled: the call 182 -> 178 us, the
            // compaction behind it 51 -> 47)
            const pard_v4i d4_ = __builtin_nontemporal_load(reinterpret_cast<const pard_v4i*>(A.deadline + lo_s + base));
            const pard_v4i s4_ = __builtin_nontemporal_load(reinterpret_cast<const pard_v4i*>(A.stage + lo_s + base));
            const int4 d4 = make_int4(d4_.x, d4_.y, d4_.z, d4_.w), s4 = make_int4(s4_.x, s4_.y, s4_.z, s4_.w);
            dl[g][0] = d4.x; dl[g][1] = d4.y; dl[g][2] = d4.z; dl[g][3] = d4.w;
            st[g][0] = s4.x; st[g][1] = s4.y; st[g][2] = s4.z; st[g][3] = s4.w;
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const bool ok = live(base + c);
                dl[g][c] = ok ? A.deadline[lo_s + base + c] : 0;
                st[g][c] = ok ? A.stage[lo_s + base + c] : 0;
            }
        }
    }
    {
        uint4* z = reinterpret_cast<uint4*>(L.cnt32);
        for (int i = tid; i < (kCntWords + 4) / 4; i += T) z[i] = make_uint4(0, 0, 0, 0);
        const uint32_t* src = reinterpret_cast<const uint32_t*>(P.recs + (int64_t)dag * S);
        uint32_t* dst = reinterpret_cast<uint32_t*>(L.recs);
        for (int i = tid; i < S * (int)(sizeof(StageRec) / 4); i += T) dst[i] = src[i];
        for (int i = tid; i < SCAP; i += T) L.down[i] = 0;
        if (tid == 0) { L.red[0] = 0xFFFFFFFFu; L.red[1] = 0u; L.slow_stages = 0u; }
        // cache in the (so far unused) index array: the DAG's latency tables and path entries
        for (int i = tid; i < S * PARD_LAT_ENTRIES; i += T) aux[i] = (uint32_t)lat_dag[i];
        if (entries_cached)
            for (int e = tid; e < n_entries; e += T)
                aux[S * PARD_LAT_ENTRIES + e] = (uint32_t)P.entry_stage[e_lo + e] | ((uint32_t)(P.entry_end[e_lo + e] - e_lo) << 8);
    }
    __syncthreads();

    // ---- order keys, snapshot-wide key range ------------------------------------
    uint32_t uk[G][4];
    uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        if (dead_group(g)) continue;
        const int base = (g * T + tid) * 4;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const bool ok = live(base + c);
            const int s = clamp_stage(st[g][c], S);
            st[g][c] = s;
            uint32_t k;
            if (P.uniform_mode == PARD_ORDER_LBF) k = (uint32_t)dl[g][c] ^ 0x80000000u;
            else if (P.uniform_mode == PARD_ORDER_HBF) k = ~((uint32_t)dl[g][c] ^ 0x80000000u);
            else {
                const int mode = P.uniform_mode >= 0 ? P.uniform_mode : (L.recs[s].mode & 0xFF);
                int32_t arr = 0;
                if (mode == PARD_ORDER_FCFS && ok) arr = A.arrival[lo_s + base + c];
                k = order_key(mode, dl[g][c], arr);
            }
            uk[g][c] = k;
            if (ok) { kmin = k < kmin ? k : kmin; kmax = k > kmax ? k : kmax; }
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const uint32_t a = __shfl_xor(kmin, off), b = __shfl_xor(kmax, off);
        kmin = a < kmin ? a : kmin;
        kmax = b > kmax ? b : kmax;
    }
    if (lane == 0) { atomicMin(&L.red[0], kmin); atomicMax(&L.red[1], kmax); }
    __syncthreads();

    // ---- 2. buckets -------------------------------------------------------------
    // Conceptually comp = (key - min) << 13 | index, bucket = stage * NB + (comp >> shift),
    // and the bits of comp below `shift` (its low part) order the requests inside a bucket.
    const uint32_t umin = L.red[0];
    const uint32_t urange = m > 0 ? L.red[1] - umin : 0u;
    int log2nb = 0;
    while ((2 << log2nb) * S <= kBuckets) ++log2nb;             // NB = largest power of two with S*NB <= kBuckets
    const int cbits = kIdxBits + (urange ? 32 - __clz((int)urange) : 0);
    const int shift = cbits > log2nb ? cbits - log2nb : 0;
    const bool key_split = shift >= kIdxBits;                   // bucket id takes key bits only
    const int ksh = key_split ? shift - kIdxBits : 0;           // key bits left below the bucket id
    const bool wide = shift > 32;                               // low part does not fit one word

    uint32_t bs[G][4];                       // bucket | slot << 16
#pragma unroll
    for (int g = 0; g < G; ++g) {
        if (dead_group(g)) continue;
        const int base = (g * T + tid) * 4;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            bs[g][c] = 0;
            if (live(base + c)) {
                const uint32_t rel = uk[g][c] - umin, me = (uint32_t)(base + c);
                uint32_t b;
                if (key_split) {
                    b = rel >> ksh;
                    if (!wide) uk[g][c] = ((rel & ((1u << ksh) - 1u)) << kIdxBits) | me;
                } else {
                    b = (rel << (kIdxBits - shift)) | (me >> shift);
                    uk[g][c] = me & ((1u << shift) - 1u);
                }
                b += (uint32_t)st[g][c] << log2nb;
                const uint32_t old = atomicAdd(&L.cnt32[b >> 1], 1u << ((b & 1u) << 4));
                bs[g][c] = b | (((old >> ((b & 1u) << 4)) & 0xFFFFu) << 16);
            }
        }
    }
    __syncthreads();

    // ---- exclusive scan of the 16-bit counters, in place ----------------------------
    {
        uint32_t w[CW];
        uint32_t sum = 0;
#pragma unroll
        for (int i = 0; i < CW / 2; ++i) {
            const uint2 v = reinterpret_cast<const uint2*>(L.cnt32)[tid * (CW / 2) + i];
            w[2 * i] = v.x; w[2 * i + 1] = v.y;
            sum += v.x + v.y;
        }
        const uint32_t tot = (sum & 0xFFFFu) + (sum >> 16);
        uint32_t inc = tot;
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
            const uint32_t t = __shfl_up(inc, off);
            if (lane >= off) inc += t;
        }
        if (lane == kWave - 1) L.wave_tot[wave] = inc;
        __syncthreads();
        uint32_t run = inc - tot;
        for (int i = 0; i < wave; ++i) run += L.wave_tot[i];
#pragma unroll
        for (int i = 0; i < CW; ++i) {
            const uint32_t l16 = w[i] & 0xFFFFu, h16 = w[i] >> 16;
            w[i] = run | ((run + l16) << 16);
            run += l16 + h16;
        }
#pragma unroll
        for (int i = 0; i < CW / 2; ++i)
            reinterpret_cast<uint2*>(L.cnt32)[tid * (CW / 2) + i] = make_uint2(w[2 * i], w[2 * i + 1]);
        if (tid == 0) L.cnt32[kCntWords] = (uint32_t)m;         // start of the bucket past the last one
    }
    __syncthreads();

    // ---- 3. queue starts, full-queue costs; scatter the low parts by bucket -----------
    const uint16_t* start16 = reinterpret_cast<const uint16_t*>(L.cnt32);
    if (tid < S) {
        const int a = start16[tid << log2nb];
        const int b = start16[(tid + 1) << log2nb];
        L.seg_start[tid] = a;
        if (tid == S - 1) L.seg_start[S] = m;
        L.cfull[tid] = stage_cost(L.recs[tid], (uint32_t)(b - a), lat_dag + tid * PARD_LAT_ENTRIES);
        const StageRec& r = L.recs[tid];
        L.quick[tid][0] = (uint32_t)r.B - 1u;
        L.quick[tid][1] = __float_as_uint(r.rcpB);
        L.quick[tid][2] = __float_as_uint(r.rcpW);
        L.quick[tid][3] = r.aW;
        L.quick[tid][4] = r.bW;
        L.quick[tid][5] = (uint32_t)a;
        if (!(r.mode & kStageFast)) L.slow_stages = 1u;
    }
    uint32_t se[G][4];                       // bucket start (13 bits) | bucket size - 1 (13 bits) | stage << 26
#pragma unroll
    for (int g = 0; g < G; ++g) {
        if (dead_group(g)) continue;
        const int base = (g * T + tid) * 4;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            se[g][c] = 0;
            if (live(base + c)) {
                const uint32_t b = bs[g][c] & 0xFFFFu, slot = bs[g][c] >> 16;
                const uint32_t s0 = start16[b], e0 = start16[b + 1];
                L.low[s0 + slot] = uk[g][c];
                if (wide) L.idx[s0 + slot] = (uint16_t)(base + c);
                se[g][c] = s0 | ((e0 - s0 - 1u) << 13) | ((b >> log2nb) << 26);
            }
        }
    }
    __syncthreads();

    // ---- 4. downstream maximum per stage over the path CSR (or as given) ---------------
    if (A.sub) {
        if (tid < S) {
            const int64_t v = A.sub[(int64_t)u * S + tid];
            L.down[tid] = v < 0 ? 0ull : ((uint64_t)v < kCostCap ? (unsigned long long)v : (unsigned long long)kCostCap);
        }
    } else if (entries_cached && !wide) {
        const uint32_t* ent = aux + S * PARD_LAT_ENTRIES;         // stage | (end of the entry's path) << 8
        for (int e = tid; e < n_entries; e += T) {
            const uint32_t me = ent[e];
            const int end = (int)(me >> 8);
            unsigned long long sum = 0;
            for (int t = e + 1; t < end; ++t) sum += L.cfull[ent[t] & 0xFFu];
            atomicMax(&L.down[me & 0xFFu], sum);
        }
    } else {
        for (int e = e_lo + tid; e < e_lo + n_entries; e += T) {
            const int end = P.entry_end[e];
            unsigned long long sum = 0;
            for (int t = e + 1; t < end; ++t) sum += L.cfull[P.entry_stage[t]];
            atomicMax(&L.down[P.entry_stage[e]], sum);
        }
    }
    // ---- exact rank inside the bucket ----------------------------------------------------
    if (!wide) {
        // the first four bucket mates of every request in straight-line code (their LDS reads
        // overlap; reads past the end of a short bucket are masked), longer buckets after that
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (dead_group(g)) continue;
            uint32_t part[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t s0 = se[g][c] & 0x1FFFu, more = (se[g][c] >> 13) & 0x1FFFu;   // bucket size - 1
                const uint32_t k = uk[g][c];
                const uint32_t a0 = L.low[s0], a1 = L.low[s0 + 1], a2 = L.low[s0 + 2], a3 = L.low[s0 + 3];
                part[c] = (uint32_t)(a0 < k) + (uint32_t)((more >= 1u) & (a1 < k)) +
                          (uint32_t)((more >= 2u) & (a2 < k)) + (uint32_t)((more >= 3u) & (a3 < k));
            }
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t s0 = se[g][c] & 0x1FFFu, more = (se[g][c] >> 13) & 0x1FFFu;
                uint32_t less = part[c];
                if (more >= 4u) {
                    const uint32_t k = uk[g][c];
                    for (uint32_t j = s0 + 4; j <= s0 + more; ++j) less += (uint32_t)(L.low[j] < k);
                }
                se[g][c] = (s0 + less) | (se[g][c] & 0xFC000000u);   // final queue slot | stage << 26
            }
        }
    } else {
        const int base0 = tid * 4;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (dead_group(g)) continue;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (live(g * T * 4 + base0 + c)) {
                    const uint32_t s0 = se[g][c] & 0x1FFFu, e0 = s0 + ((se[g][c] >> 13) & 0x1FFFu) + 1u;
                    const uint32_t k = uk[g][c], me = (uint32_t)(g * T * 4 + base0 + c);
                    uint32_t less = 0;
                    for (uint32_t j = s0; j < e0; ++j) {
                        const uint32_t kj = L.low[j], ij = L.idx[j];
                        less += (uint32_t)((kj < k) | ((kj == k) & (ij < me)));
                    }
                    se[g][c] = (s0 + less) | (se[g][c] & 0xFC000000u);
                }
            }
        }
    }
    __syncthreads();                         // bucket starts are no longer needed; down[] is complete
    uint16_t* ord_l = reinterpret_cast<uint16_t*>(L.cnt32);
#pragma unroll
    for (int g = 0; g < G; ++g) {
        if (dead_group(g)) continue;
        const int base = (g * T + tid) * 4;
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (live(base + c)) ord_l[se[g][c] & 0x1FFFu] = (uint16_t)(base + c);
    }

    if (CONSISTENT) {
        // ---- 5'. decisions in queue order, positions = kept requests ahead -------------------
        // deadlines by queue slot (L.low is free: every read of the rank phase is behind the barrier above)
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (dead_group(g)) continue;
            const int base = (g * T + tid) * 4;
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (live(base + c)) L.low[se[g][c] & 0x1FFFu] = (uint32_t)dl[g][c];
        }
        __syncthreads();
        for (int k = wave; k < S; k += T / kWave) {            // one wave per queue
            const int s0 = L.seg_start[k], s1 = L.seg_start[k + 1];
            const unsigned long long dn = L.down[k];
            // the DAG's latency tables sit in LDS unless the wide case took that array back
            const int32_t* lat_row = wide ? lat_dag + k * PARD_LAT_ENTRIES : reinterpret_cast<const int32_t*>(aux) + k * PARD_LAT_ENTRIES;
            const int32_t order = L.recs[k].mode & 0xFF;
            // A latency table that never falls up to the batch size makes the cost rise with the position, so the
            // positions at which a request is still in time form a prefix; in a queue ordered by deadline the chain
            // of decisions then has a closed form per 64 requests (below).  Anything else is iterated.
            const bool falls = lane + 1 < L.recs[k].B && lat_row[lane + 1] < lat_row[lane];
            const bool closed = __ballot(falls) == 0ull && order != PARD_ORDER_FCFS;
            uint32_t kept = 0;                                  // kept requests of this queue so far (same in every lane)
            bool cut = false;                                   // high budget first: a request has been dropped already
            for (int first = s0; first < s1; first += kWave) {
                const int j = first + lane;
                const bool ok = j < s1;
                const int32_t deadline = ok ? (int32_t)L.low[j] : 0;
                unsigned long long keep;
                int32_t est = 0;
                uint8_t drp = 0;
                if (closed && order == PARD_ORDER_LBF) {
                    // Lane l evaluates position kept + l.  Budgets rise along the queue, so does the number c of
                    // positions (counted from `kept`) a request is in time at, and the recurrence
                    // a' = min(a + 1, c) unrolls to a_i = min(i, i - 1 + min over i' < i of (c_i' - i')).
                    const uint32_t at = kept + (uint32_t)lane < (uint32_t)(CAP - 1) ? kept + (uint32_t)lane : (uint32_t)(CAP - 1);
                    const uint64_t e64 = stage_cost_short(L.recs[k], at, lat_row) + dn;
                    const int32_t est_at = e64 > (uint64_t)kInt32Max ? kInt32Max : (int32_t)e64;
                    const int64_t fin = (int64_t)now + (int64_t)e64;
                    const int32_t end_at = fin > (int64_t)kInt32Max ? kInt32Max : (int32_t)fin;     // late iff end_at > deadline
                    // c: positions kept .. kept + c - 1 are in time (c <= 64); end_at rises with the lane, so first the
                    // blocks of eight positions that fit as a whole (their last lane's value, read as a scalar), then
                    // three steps inside the next block
                    int c = 0;
#pragma unroll
                    for (int b = 0; b < kWave / 8; ++b) c += __builtin_amdgcn_readlane(end_at, 8 * b + 7) <= deadline ? 8 : 0;
#pragma unroll
                    for (int step = 4; step >= 1; step >>= 1) {
                        const int32_t probe = __shfl(end_at, (c + step - 1) & (kWave - 1));
                        if (c < kWave && probe <= deadline) c += step;
                    }
                    const int32_t least = wave_exclusive_min(c - lane);        // min over lower lanes, INT32_MAX for lane 0
                    int a = lane;
                    if (lane > 0 && lane - 1 + (int64_t)least < (int64_t)a) a = lane - 1 + least;
                    est = __shfl(est_at, a);
                    drp = (ok && a < c) ? 0 : 1;
                    keep = __ballot(ok && a < c);
                } else if (closed) {
                    // High budget first: budgets fall along the queue, so once a request is late at its plain
                    // position every later one is late at that same position.
                    const uint32_t at = kept + (cut ? 0u : (uint32_t)lane);
                    finish_request(stage_cost_short(L.recs[k], at < (uint32_t)(CAP - 1) ? at : (uint32_t)(CAP - 1), lat_row) + dn,
                                   now, deadline, est, drp);
                    keep = 0ull;
                    if (!cut) {
                        const unsigned long long late = __ballot(ok && drp != 0);
                        const int f = late ? __builtin_ctzll(late) : kWave;    // the first late request of the chunk
                        keep = __ballot(ok && lane < f);
                        const int32_t est_cut = __shfl(est, f < kWave ? f : 0);
                        if (lane >= f) { est = est_cut; drp = 1; }
                        cut = late != 0ull;
                    } else {
                        drp = 1;
                    }
                } else {
                    // Guess that all 64 are kept, evaluate everybody at the position that guess implies,
                    // take the decisions as the next guess: after t rounds the first t lanes are final,
                    // and a guess that reproduces itself is the in-order result.
                    keep = __ballot(ok);
                    for (int round = 0; round <= kWave; ++round) {
                        const uint32_t ahead = kept + __builtin_amdgcn_mbcnt_hi((uint32_t)(keep >> 32),
                                                          __builtin_amdgcn_mbcnt_lo((uint32_t)keep, 0u));
                        finish_request(stage_cost_short(L.recs[k], ahead, lat_row) + dn, now, deadline, est, drp);
                        const unsigned long long next = __ballot(ok && drp == 0);
                        if (next == keep) break;
                        keep = next;
                    }
                }
                if (ok) L.low[j] = (uint32_t)est | ((uint32_t)drp << 31);
                kept += (uint32_t)__popcll(keep);
            }
        }
        __syncthreads();
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (dead_group(g)) continue;
            const int base = (g * T + tid) * 4;
            int32_t est[4];
            uint8_t drp[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t v = live(base + c) ? L.low[se[g][c] & 0x1FFFu] : 0u;
                est[c] = (int32_t)(v & 0x7FFFFFFFu);
                drp[c] = (uint8_t)(v >> 31);
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
    }

    // ---- 5. estimate and drop decision, request order ---------------------------------
    const bool quick = !wide && L.slow_stages == 0u;          // every stage admits the exact short-queue form
#pragma unroll
    for (int g = 0; g < (CONSISTENT ? 0 : G); ++g) {
        if (dead_group(g)) continue;
        const int base = (g * T + tid) * 4;
        int32_t est[4];
        uint8_t drp[4];
        asm volatile("" ::: "memory");           // one group of four requests at a time (register pressure)
        if (quick) {
            // straight-line: stage_cost_short() with the per-stage constants and the latency table in LDS
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t k = se[g][c] >> 26;
                const uint4 qa = *reinterpret_cast<const uint4*>(&L.quick[k][0]);     // B-1, 1/B, 1/W, aW
                const uint2 qb = *reinterpret_cast<const uint2*>(&L.quick[k][4]);     // bW, queue start
                const unsigned long long dn = L.down[k];
                const uint32_t pos = (se[g][c] & 0x1FFFu) - qb.y;
                const uint32_t q = (uint32_t)(((float)(pos + qa.x) + 0.5f) * __uint_as_float(qa.y));
                const uint32_t p = __umul24(q, qb.x);
                const uint32_t wait = __umul24(q, qa.w) + (uint32_t)(((float)p + 0.5f) * __uint_as_float(qa.z));
                const uint32_t seen = pos < qa.x ? pos : qa.x;
                const uint64_t e64 = (uint64_t)wait + aux[k * PARD_LAT_ENTRIES + seen] + dn;
                finish_request(e64, now, dl[g][c], est[c], drp[c]);
            }
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                est[c] = 0;
                drp[c] = 0;
                if (live(base + c)) {
                    const int k = (int)(se[g][c] >> 26);
                    const uint32_t pos = (se[g][c] & 0x1FFFu) - (uint32_t)L.seg_start[k];
                    const uint64_t cost = stage_cost_short(L.recs[k], pos, lat_dag + k * PARD_LAT_ENTRIES);
                    finish_request(cost + L.down[k], now, dl[g][c], est[c], drp[c]);
                }
            }
        }
        if (A.kept) {                        // survivor staging below: a dropped request's queue slot carries the decision
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (live(base + c) && drp[c]) ord_l[se[g][c] & 0x1FFFu] = (uint16_t)((uint32_t)(base + c) | 0x8000u);
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

    // ---- queue order and queue offsets out ----------------------------------------------
    // (an entry of ord_l[] is local index | drop << 15; the drop bit is only set when survivors are staged)
    uint32_t ent[G][4];
    const int32_t b32 = (int32_t)lo_s;
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
        for (int c = 0; c < 4; ++c) ent[g][c] = 0x8000u;         // not a slot: counts as dropped below
        if (dead_group(g)) continue;
        const int base = (g * T + tid) * 4;
        // queue slot q sits at order[lo + q] = order[lo_s + (q + off)]: the same shifted groups of four;
        // its entry is the request with local index ord_l[q], i.e. request lo_s + ord_l[q]
        if (whole(base)) {
            if (off == 0) {
                const uint2 o = *reinterpret_cast<const uint2*>(ord_l + base);
                ent[g][0] = o.x & 0xFFFFu; ent[g][1] = o.x >> 16;
                ent[g][2] = o.y & 0xFFFFu; ent[g][3] = o.y >> 16;
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c) ent[g][c] = ord_l[base - off + c];
            }
            *reinterpret_cast<int4*>(A.order + lo_s + base) =
                make_int4(b32 + (int32_t)(ent[g][0] & 0x7FFFu), b32 + (int32_t)(ent[g][1] & 0x7FFFu),
                          b32 + (int32_t)(ent[g][2] & 0x7FFFu), b32 + (int32_t)(ent[g][3] & 0x7FFFu));
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (live(base + c)) {
                    ent[g][c] = ord_l[base - off + c];
                    A.order[lo_s + base + c] = b32 + (int32_t)(ent[g][c] & 0x7FFFu);
                }
        }
    }
    if (tid < S) A.seg_ptr[(int64_t)u * S + tid] = (int32_t)lo + L.seg_start[tid];
    if (u == P.K - 1 && tid == 0) A.seg_ptr[(int64_t)P.K * S] = (int32_t)(lo + m);
    if (CONSISTENT || !A.kept) return;

    // ---- survivors of this snapshot in queue order, staged at the snapshot's own place ----------
    // (the compaction's last kernel moves them to their final place once the counts of all snapshots are known)
    // Queue slots run group-major here: group g of thread t holds the shifted slots [(g T + t) 4, +4).
    static_assert(G <= 4, "two words of two 16-bit counts");
    uint32_t keep[G];
    uint32_t c01 = 0, c23 = 0;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        keep[g] = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) keep[g] |= ((ent[g][c] >> 15) ^ 1u) << c;
        const uint32_t cnt = (uint32_t)__popc(keep[g]);
        if (g < 2) c01 |= cnt << (16 * g); else c23 |= cnt << (16 * (g - 2));
    }
    const uint32_t i01 = wave_inclusive_sum(c01), i23 = wave_inclusive_sum(c23);
    if (lane == kWave - 1) { L.kept_tot[wave][0] = i01; L.kept_tot[wave][1] = i23; }
    __syncthreads();
    uint32_t tot01 = 0, tot23 = 0, bef01 = 0, bef23 = 0;       // all waves / the waves before this one
#pragma unroll
    for (int w = 0; w < T / kWave; ++w) {
        const uint32_t a = L.kept_tot[w][0], b = L.kept_tot[w][1];
        tot01 += a; tot23 += b;
        if (w < wave) { bef01 += a; bef23 += b; }
    }
    const uint32_t gt[4] = {tot01 & 0xFFFFu, tot01 >> 16, tot23 & 0xFFFFu, tot23 >> 16};
    const uint32_t total = gt[0] + gt[1] + gt[2] + gt[3];
    const uint32_t x01 = bef01 + i01 - c01, x23 = bef23 + i23 - c23;
    int32_t* stage_at = A.staged + lo + staging_shift(u, (uint32_t)m, total);
    uint32_t* grp = L.low;                   // free by now: per group of four slots the kept slots before it | keep bits << 14
    uint32_t groups_before = 0;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        uint32_t o = groups_before + (g < 2 ? (x01 >> (16 * g)) & 0xFFFFu : (x23 >> (16 * (g - 2))) & 0xFFFFu);
        groups_before += gt[g];
        grp[g * T + tid] = o | (keep[g] << 14);
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (keep[g] & (1u << c)) { stage_at[o] = b32 + (int32_t)(ent[g][c] & 0x7FFFu); ++o; }
    }
    __syncthreads();
    for (int k = tid; k < S; k += T) {
        const int ps = L.seg_start[k] + off;             // the queue's first slot in this layout
        uint32_t before = total;
        if (ps < m_s) {
            const uint32_t v = grp[ps >> 2];
            before = (v & 0x3FFFu) + (uint32_t)__popc((v >> 14) & ((1u << (ps & 3)) - 1u));
        }
        A.loc_ptr[(int64_t)u * S + k] = (int32_t)before;
    }
    if (tid == 0) A.kept[u] = total;
}

template <int T, int CAP, int SCAP, bool CONSISTENT>
__global__ __launch_bounds__(T, 4) void fused_snapshot_kernel(FusedArgs A) {
    constexpr int kCap = CAP;
    __shared__ SnapshotLds<CAP, SCAP> L;
    const int u = blockIdx.x;
    // (the mark and the snapshot's bounds are asked for together: one wait instead of two for a marked snapshot)
    const uint32_t marked = A.todo ? A.todo[u] : 1u;
    int64_t lo = A.snap_ptr[u], hi = A.snap_ptr[u + 1];
    if (marked == 0u) return;                    // already done by the kernel for snapshots that come in queue order
    const int64_t n = A.n;
    // snapshot bounds, made safe whatever snap_ptr holds
    if (lo < 0) lo = 0;
    if (lo > n) lo = n;
    if (hi > n) hi = n;
    int64_t m64 = hi - lo;
    if (m64 < 0) m64 = 0;
    const int limit = A.cap < kCap ? A.cap : kCap;
    if (m64 > limit) {
        m64 = limit;
        if (threadIdx.x == 0) atomicOr(A.status, kStatusSnapshotTooLarge);
    }
    const int m = (int)m64;
    const uintptr_t bits = reinterpret_cast<uintptr_t>(A.deadline) | reinterpret_cast<uintptr_t>(A.stage) |
                           reinterpret_cast<uintptr_t>(A.est) | reinterpret_cast<uintptr_t>(A.order) |
                           (reinterpret_cast<uintptr_t>(A.drop) << 2);
    // 16-byte accesses need aligned arrays; the snapshot's own start is taken care of by shifting the
    // local indices by lo mod 4, as long as the shifted snapshot still fits the capacity
    const int shift = (int)(lo & 3);
    const bool aligned = (bits & 15) == 0 && m + shift <= kCap;
    const int off = aligned ? shift : 0;
    if (m == kCap && aligned && off == 0) snapshot_body<T, CAP, SCAP, true, CONSISTENT>(A, L, u, lo, m, true, 0);
    else snapshot_body<T, CAP, SCAP, false, CONSISTENT>(A, L, u, lo, m, aligned, off);
}

template <int CAP, int T, int SCAP>
void launch_stages(const FusedArgs& a, hipStream_t stream) {
    if (a.consistent) fused_snapshot_kernel<T, CAP, SCAP, true><<<dim3((unsigned)a.plan.K), dim3(T), 0, stream>>>(a);
    else fused_snapshot_kernel<T, CAP, SCAP, false><<<dim3((unsigned)a.plan.K), dim3(T), 0, stream>>>(a);
}

template <int CAP, int T>
void launch_capacity(const FusedArgs& a, hipStream_t stream) {
    // at the full capacity the request arrays dominate the LDS and two workgroups fit either way
    if constexpr (CAP < PARD_FUSED_SNAPSHOT_CAPACITY) {
        if (a.plan.S <= kFewStages) return launch_stages<CAP, T, kFewStages>(a, stream);
        if (a.plan.S <= kSomeStages) return launch_stages<CAP, T, kSomeStages>(a, stream);
    }
    launch_stages<CAP, T, PARD_MAX_STAGES>(a, stream);
}

}  // namespace

hipError_t launch_fused(const FusedArgs& args, hipStream_t stream) {
    FusedArgs a = args;
    if (wave_path_covers(a)) { a.todo = nullptr; return launch_wave(a, stream); }      // a few dozen requests per snapshot: one wave each
    // Snapshots in queue order are finished by the kernel made for them; it marks the others in todo[],
    // and the general kernel below then works on the marked ones only (every other workgroup returns at once).
    if (presorted_path_covers(a)) {
        const hipError_t e = launch_presorted(a, stream);
        if (e != hipSuccess) return e;
    } else {
        a.todo = nullptr;
    }
    // the smallest workgroup whose capacity covers the promised snapshot size
    if (a.cap <= 256) launch_capacity<256, 64>(a, stream);
    else if (a.cap <= 512) launch_capacity<512, 64>(a, stream);
    else if (a.cap <= 1024) launch_capacity<1024, 128>(a, stream);
    else if (a.cap <= 2048) launch_capacity<2048, 128>(a, stream);
    else if (a.cap <= 4096) launch_capacity<4096, 256>(a, stream);
    else launch_capacity<PARD_FUSED_SNAPSHOT_CAPACITY, 512>(a, stream);
    return hipGetLastError();
}

}  // namespace pard
