// On-chip path: one workgroup evaluates one whole snapshot (up to 8192 queued requests)
// with a single read of the inputs and a single write of the outputs.
//
// Per snapshot (paper Section 3.2 Eq.(1),(2),(4), DAG maximum; Section 3.3 ordering):
//   1. load deadline/stage (arrival for FCFS stages), form the order key
//   2. bucket every request by (stage, leading bits of key.index) with LDS counters;
//      the bucket order is the queue order, so an exclusive scan of the counters gives
//      every bucket's first queue slot and every stage's queue start and length
//   3. scatter (key, index) into LDS by bucket; a request's exact rank is its bucket
//      start plus the number of bucket mates with a smaller (key, index)
//   4. per stage: cost at full queue length; per path entry: downstream suffix sum,
//      maximum per stage (the path CSR is walked here)
//   5. per request: own-stage cost at its queue position + downstream maximum,
//      drop decision; outputs leave in request order, the queue order via LDS.
//
// Why buckets instead of radix passes: the vector ALU, not HBM, is what limits a sort of
// 8192 keys per workgroup at this data rate (about 130 lane-instructions per request at
// full HBM speed).  A stable 8-bit radix pass costs ~70 of them per key per pass.  One
// bucketing pass with ~0.7 requests per bucket and a compare loop over bucket mates costs
// less than one radix pass.  Appending the request index below the key makes equal keys
// spread over buckets too, so heavy ties stay cheap; only a strongly clustered key
// distribution degrades to many compares per request (still exact).
#include "pard_device.hpp"

namespace pard {

namespace {

constexpr int kCap = PARD_FUSED_SNAPSHOT_CAPACITY;   // requests per snapshot, at most
constexpr int kIdxBits = 13;                         // 8192 = 2^13 local indices
constexpr int kBuckets = 12288;                      // 16-bit counters, two per LDS word
constexpr int kCntWords = kBuckets / 2;

static_assert(kCap == (1 << kIdxBits), "local index width");

template <int T>
__global__ __launch_bounds__(T) void fused_snapshot_kernel(FusedArgs A) {
    constexpr int G = kCap / (4 * T);       // groups of 4 consecutive requests per thread
    constexpr int NW = T / kWave;
    constexpr int CW = kCntWords / T;       // counter words scanned per thread
    static_assert(G >= 1 && CW >= 1 && kCntWords % T == 0, "shape");

    __shared__ __align__(16) uint32_t cnt32[kCntWords + 4];       // bucket counters, then bucket starts; later the queue order
    __shared__ __align__(16) uint32_t key_l[kCap];
    __shared__ __align__(16) uint16_t idx_l[kCap];
    __shared__ StageRec recs[PARD_MAX_STAGES];
    __shared__ unsigned long long cfull[PARD_MAX_STAGES];
    __shared__ unsigned long long down[PARD_MAX_STAGES];
    __shared__ int32_t seg_start[PARD_MAX_STAGES + 1];
    __shared__ uint32_t wave_tot[NW];
    __shared__ uint32_t red[2];

    const PlanDev& P = A.plan;
    const int64_t n = A.n;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int u = blockIdx.x;
    const int S = P.S;
    const int dag = P.shared ? 0 : u;

    // snapshot bounds, made safe whatever snap_ptr holds
    int64_t lo64 = A.snap_ptr[u], hi64 = A.snap_ptr[u + 1];
    if (lo64 < 0) lo64 = 0;
    if (lo64 > n) lo64 = n;
    if (hi64 > n) hi64 = n;
    int64_t m64 = hi64 - lo64;
    if (m64 < 0) m64 = 0;
    const int limit = A.cap < kCap ? A.cap : kCap;
    if (m64 > limit) {
        m64 = limit;
        if (tid == 0) atomicOr(A.status, kStatusSnapshotTooLarge);
    }
    const int m = (int)m64;
    const int64_t lo = lo64;
    const bool aligned = (lo & 3) == 0;

    // ---- 1. loads (issued first), LDS initialisation meanwhile ---------------
    int32_t dl[G][4], st[G][4];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const int base = (g * T + tid) * 4;
        if (aligned && base + 3 < m) {
            int4 d4 = *reinterpret_cast<const int4*>(A.deadline + lo + base);
            int4 s4 = *reinterpret_cast<const int4*>(A.stage + lo + base);
            dl[g][0] = d4.x; dl[g][1] = d4.y; dl[g][2] = d4.z; dl[g][3] = d4.w;
            st[g][0] = s4.x; st[g][1] = s4.y; st[g][2] = s4.z; st[g][3] = s4.w;
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const bool ok = base + c < m;
                dl[g][c] = ok ? A.deadline[lo + base + c] : 0;
                st[g][c] = ok ? A.stage[lo + base + c] : 0;
            }
        }
    }
    for (int i = tid; i < kCntWords + 4; i += T) cnt32[i] = 0;
    {
        const uint32_t* src = reinterpret_cast<const uint32_t*>(P.recs + (int64_t)dag * S);
        uint32_t* dst = reinterpret_cast<uint32_t*>(recs);
        for (int i = tid; i < S * 8; i += T) dst[i] = src[i];
    }
    if (tid < PARD_MAX_STAGES) down[tid] = 0;
    if (tid == 0) { red[0] = 0xFFFFFFFFu; red[1] = 0u; }
    __syncthreads();

    // ---- order keys, snapshot-wide key range ------------------------------------
    uint32_t uk[G][4];
    uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const int base = (g * T + tid) * 4;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const bool ok = base + c < m;
            const int s = clamp_stage(st[g][c], S);
            st[g][c] = s;
            const int mode = P.uniform_mode >= 0 ? P.uniform_mode : recs[s].mode;
            int32_t arr = 0;
            if (P.any_fcfs && mode == PARD_ORDER_FCFS && ok) arr = A.arrival[lo + base + c];
            const uint32_t k = order_key(mode, dl[g][c], arr);
            uk[g][c] = k;
            if (ok) { kmin = k < kmin ? k : kmin; kmax = k > kmax ? k : kmax; }
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        uint32_t a = __shfl_xor(kmin, off), b = __shfl_xor(kmax, off);
        kmin = a < kmin ? a : kmin;
        kmax = b > kmax ? b : kmax;
    }
    if (lane == 0) { atomicMin(&red[0], kmin); atomicMax(&red[1], kmax); }
    __syncthreads();

    // ---- 2. buckets -------------------------------------------------------------
    const uint32_t umin = red[0];
    const uint32_t urange = m > 0 ? red[1] - umin : 0u;
    int log2nb = 0;
    while ((2 << log2nb) * S <= kBuckets) ++log2nb;             // NB = largest power of two with S*NB <= kBuckets
    const uint64_t crange = ((uint64_t)urange << kIdxBits) | (uint64_t)(kCap - 1);
    const int cbits = 64 - __clzll((long long)crange);
    const int shift = cbits > log2nb ? cbits - log2nb : 0;

    uint32_t bs[G][4];                       // bucket | slot << 16
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const int base = (g * T + tid) * 4;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            bs[g][c] = 0;
            if (base + c < m) {
                const uint64_t comp = ((uint64_t)(uk[g][c] - umin) << kIdxBits) | (uint32_t)(base + c);
                const uint32_t b = ((uint32_t)st[g][c] << log2nb) + (uint32_t)(comp >> shift);
                const uint32_t old = atomicAdd(&cnt32[b >> 1], (b & 1u) ? 0x10000u : 1u);
                const uint32_t slot = (b & 1u) ? (old >> 16) : (old & 0xFFFFu);
                bs[g][c] = b | (slot << 16);
            }
        }
    }
    __syncthreads();

    // ---- exclusive scan of the 16-bit counters, in place ----------------------------
    {
        uint32_t w[CW];
        uint32_t sum = 0;
#pragma unroll
        for (int i = 0; i < CW; ++i) { w[i] = cnt32[tid * CW + i]; sum += w[i]; }
        const uint32_t tot = (sum & 0xFFFFu) + (sum >> 16);
        uint32_t inc = tot;
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
            uint32_t t = __shfl_up(inc, off);
            if (lane >= off) inc += t;
        }
        if (lane == kWave - 1) wave_tot[wave] = inc;
        __syncthreads();
        uint32_t run = inc - tot;
        for (int i = 0; i < wave; ++i) run += wave_tot[i];
#pragma unroll
        for (int i = 0; i < CW; ++i) {
            const uint32_t l16 = w[i] & 0xFFFFu, h16 = w[i] >> 16;
            cnt32[tid * CW + i] = run | ((run + l16) << 16);
            run += l16 + h16;
        }
        if (tid == 0) cnt32[kCntWords] = (uint32_t)m;           // start of the bucket past the last one
    }
    __syncthreads();

    // ---- 3. queue starts, full-queue costs; scatter (key, index) by bucket -----------
    const uint16_t* start16 = reinterpret_cast<const uint16_t*>(cnt32);
    if (tid < S) {
        const int a = start16[tid << log2nb];
        const int b = start16[(tid + 1) << log2nb];
        seg_start[tid] = a;
        if (tid == S - 1) seg_start[S] = m;
        cfull[tid] = stage_cost(recs[tid], (uint32_t)(b - a), P.lat + ((int64_t)dag * S + tid) * PARD_LAT_ENTRIES);
    }
    uint32_t se[G][4];                       // bucket start | bucket end << 16
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const int base = (g * T + tid) * 4;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            se[g][c] = 0;
            if (base + c < m) {
                const uint32_t b = bs[g][c] & 0xFFFFu, slot = bs[g][c] >> 16;
                const uint32_t s0 = start16[b], e0 = start16[b + 1];
                key_l[s0 + slot] = uk[g][c];
                idx_l[s0 + slot] = (uint16_t)(base + c);
                se[g][c] = s0 | (e0 << 16);
            }
        }
    }
    __syncthreads();

    // ---- 4. downstream maximum per stage over the path CSR ---------------------------
    {
        const int e_lo = P.dag_entry_ptr[dag], e_hi = P.dag_entry_ptr[dag + 1];
        for (int e = e_lo + tid; e < e_hi; e += T) {
            const int end = P.entry_end[e];
            unsigned long long sum = 0;
            for (int t = e + 1; t < end; ++t) sum += cfull[P.entry_stage[t]];
            atomicMax(&down[P.entry_stage[e]], sum);
        }
    }
    // ---- exact rank inside the bucket; queue order into LDS (reuses cnt32) -----------
    uint16_t* ord_l = reinterpret_cast<uint16_t*>(cnt32);
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const int base = (g * T + tid) * 4;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (base + c < m) {
                const uint32_t s0 = se[g][c] & 0xFFFFu, e0 = se[g][c] >> 16;
                const uint32_t k = uk[g][c], me = (uint32_t)(base + c);
                uint32_t less = 0;
                if (e0 - s0 > 1) {
                    for (uint32_t j = s0; j < e0; ++j) {
                        const uint32_t kj = key_l[j], ij = idx_l[j];
                        less += (kj < k) | ((kj == k) & (ij < me));
                    }
                }
                se[g][c] = s0 + less;        // final queue slot inside the snapshot
            }
        }
    }
    __syncthreads();                         // every bucket start has been read; cnt32 is free
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const int base = (g * T + tid) * 4;
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (base + c < m) ord_l[se[g][c]] = (uint16_t)(base + c);
    }

    // ---- 5. estimate and drop decision, request order ---------------------------------
    const int32_t now = A.now[u];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const int base = (g * T + tid) * 4;
        int32_t est[4];
        uint8_t drp[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            est[c] = 0;
            drp[c] = 0;
            if (base + c < m) {
                const int k = st[g][c];
                const uint32_t pos = se[g][c] - (uint32_t)seg_start[k];
                const uint64_t e64 = stage_cost(recs[k], pos, P.lat + ((int64_t)dag * S + k) * PARD_LAT_ENTRIES) + down[k];
                finish_request(e64, now, dl[g][c], est[c], drp[c]);
            }
        }
        if (aligned && base + 3 < m) {
            *reinterpret_cast<int4*>(A.est + lo + base) = make_int4(est[0], est[1], est[2], est[3]);
            *reinterpret_cast<uchar4*>(A.drop + lo + base) = make_uchar4(drp[0], drp[1], drp[2], drp[3]);
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (base + c < m) { A.est[lo + base + c] = est[c]; A.drop[lo + base + c] = drp[c]; }
        }
    }
    __syncthreads();

    // ---- queue order and queue offsets out ----------------------------------------------
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const int base = (g * T + tid) * 4;
        if (aligned && base + 3 < m) {
            const uint2 o = *reinterpret_cast<const uint2*>(ord_l + base);
            const int32_t b32 = (int32_t)lo;
            *reinterpret_cast<int4*>(A.order + lo + base) =
                make_int4(b32 + (int32_t)(o.x & 0xFFFFu), b32 + (int32_t)(o.x >> 16),
                          b32 + (int32_t)(o.y & 0xFFFFu), b32 + (int32_t)(o.y >> 16));
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (base + c < m) A.order[lo + base + c] = (int32_t)lo + (int32_t)ord_l[base + c];
        }
    }
    if (tid < S) A.seg_ptr[(int64_t)u * S + tid] = (int32_t)lo + seg_start[tid];
    if (u == P.K - 1 && tid == 0) A.seg_ptr[(int64_t)P.K * S] = (int32_t)(lo + m);
}

}  // namespace

hipError_t launch_fused(const FusedArgs& a, hipStream_t stream) {
    constexpr int T = 512;
    fused_snapshot_kernel<T><<<dim3((unsigned)a.plan.K), dim3(T), 0, stream>>>(a);
    return hipGetLastError();
}

}  // namespace pard
