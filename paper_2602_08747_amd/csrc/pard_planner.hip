// The State Planner's part of the estimate (paper Section 3.2, Eq.(4) and "Batch wait
// estimation"): per (snapshot, stage), the latency of the modules after it,
//   L_sub = sum q_i + sum d_i + w,   maximum over the downstream DAG paths,
// with w the lambda-quantile of the aggregated batch wait time obtained by sampling the
// collected arrival process, and the ablation variants that replace w or drop terms
// (Section 5.1 baseline table, Section 5.3).  Also the queue lengths those terms depend on.
//
//   q_i = floor(ceil(n_i/B_i) * lat_i[B_i] / W_i) from the queue length, or the monitored delay
//   (linearly weighted sliding window over time-stamped delay samples, further down) when given;
//   d_i = lat_i[min(B_i, n_i+1)],  n_i queued at stage i
//   sample j, stage i: arrival a = max(samples[picks[j*S+i] mod M], 0) waits (d_i - a mod d_i) mod d_i
//   for the module's next batch (batches back to back, boundaries at multiples of d_i)
//   T_j = sum over the later stages of the path; w = rank-th smallest T_j (rank = ceil(lambda*M)).
#include "pard_device.hpp"

namespace pard {

namespace {

constexpr uint64_t kSubCap = (uint64_t)1 << 40;

// ---- queue lengths ---------------------------------------------------------------------
constexpr int kQThreads = 256;
constexpr int kQChunk = 4096;                          // requests per workgroup
constexpr int kQBins = 4096;                           // LDS counters per workgroup

__global__ void fill_zero_kernel(unsigned long long* p, int64_t count) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (int64_t)gridDim.x * blockDim.x) p[i] = 0ull;
}
__global__ void fill_zero32_kernel(int32_t* p, int64_t count) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (int64_t)gridDim.x * blockDim.x) p[i] = 0;
}

// snapshot of request r among snapshots [lo, hi]: the u with snap_ptr[u] <= r < snap_ptr[u+1]
__device__ __forceinline__ int32_t snapshot_in(const int32_t* snap_ptr, int32_t lo, int32_t hi, int64_t r) {
    int32_t a = lo, b = hi + 1;                        // answer in [a, b)
    while (b - a > 1) {
        const int32_t mid = (a + b) >> 1;
        if ((int64_t)snap_ptr[mid] <= r) a = mid; else b = mid;
    }
    return a;
}

// A workgroup counts 4096 consecutive requests.  They belong to a contiguous range of
// snapshots; when that range's (snapshot, stage) pairs fit the LDS counters, counting happens
// there (each counter replicated so that the lanes of a wave spread over copies) and only
// the non-zero sums go to global memory.
__global__ __launch_bounds__(kQThreads) void queue_lengths_kernel(int32_t K, int32_t S, int64_t n, const int32_t* stage,
                                                                  const int32_t* snap_ptr, int32_t* qlen) {
    __shared__ uint32_t bins[kQBins];
    __shared__ int32_t s_range[2];
    const int tid = threadIdx.x;
    const int64_t base = (int64_t)blockIdx.x * kQChunk;
    const int64_t end = base + kQChunk < n ? base + kQChunk : n;
    if (tid == 0) {
        s_range[0] = snapshot_in(snap_ptr, 0, K - 1, base);
        s_range[1] = snapshot_in(snap_ptr, 0, K - 1, end - 1);
    }
    __syncthreads();
    const int32_t u_lo = s_range[0], u_hi = s_range[1];
    const int64_t window = ((int64_t)u_hi - u_lo + 1) * S;
    const bool local = window <= kQBins;
    int copies = 1;                                    // power of two, copies * window <= kQBins, at most 32
    if (local) while (copies < 32 && (int64_t)copies * 2 * window <= kQBins) copies *= 2;
    if (local) for (int i = tid; i < copies * (int)window; i += kQThreads) bins[i] = 0;
    __syncthreads();
    for (int64_t r = base + tid; r < end; r += kQThreads) {
        const int32_t u = snapshot_in(snap_ptr, u_lo, u_hi, r);
        const int32_t s = clamp_stage(stage[r], S);
        if (local) atomicAdd(&bins[((u - u_lo) * S + s) * copies + (tid & (copies - 1))], 1u);
        else atomicAdd(&qlen[(int64_t)u * S + s], 1);
    }
    __syncthreads();
    if (local)
        for (int g = tid; g < (int)window; g += kQThreads) {
            uint32_t sum = 0;
            for (int c = 0; c < copies; ++c) sum += bins[g * copies + c];
            if (sum) atomicAdd(&qlen[(int64_t)u_lo * S + g], (int32_t)sum);
        }
}

// ---- downstream latency ----------------------------------------------------------------
// (snapshot, path entry) of work item b: with one shared DAG every snapshot has the same
// entries; otherwise entry e belongs to snapshot entry_dag[e].
__device__ __forceinline__ bool entry_of(const PlanDev& P, int64_t b, int32_t& u, int32_t& e) {
    if (P.shared) {
        const int64_t per = P.dag_entry_ptr[1];
        if (per <= 0 || b >= per * P.K) return false;
        u = (int32_t)(b / per);
        e = (int32_t)(b % per);
    } else {
        if (b >= P.total_entries) return false;
        e = (int32_t)b;
        u = P.entry_dag[e];
    }
    return true;
}

// q_i + d_i (clamped at 2^40 like every stage cost) and d_i of stage i with n queued
__device__ __forceinline__ void stage_terms(const PlanDev& P, int32_t u, int32_t i, const int32_t* qlen,
                                            const int32_t* qdelay, uint64_t& cost, uint32_t& dur) {
    const int64_t rec = (P.shared ? 0 : (int64_t)u * P.S) + i;
    const StageRec r = P.recs[rec];
    const int32_t q = qlen[(int64_t)u * P.S + i];
    const uint32_t n = q > 0 ? (uint32_t)q : 0u;
    const int32_t* lat_row = P.lat + rec * PARD_LAT_ENTRIES;
    dur = (uint32_t)lat_row[(n + 1u < (uint32_t)r.B ? n + 1u : (uint32_t)r.B) - 1u];
    if (qdelay) {
        const int32_t qd = qdelay[(int64_t)u * P.S + i];
        cost = (uint64_t)(qd > 0 ? (uint32_t)qd : 0u) + dur;
    } else {
        cost = stage_cost(r, n, lat_row);
    }
}

// Variants without sampling: one thread per (snapshot, path entry).
__global__ __launch_bounds__(256) void sub_simple_kernel(SubArgs A, int64_t items) {
    const int64_t b = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= items) return;
    const PlanDev& P = A.plan;
    int32_t u, e;
    if (!entry_of(P, b, u, e)) return;
    const int32_t k = P.entry_stage[e], end = P.entry_end[e];
    uint64_t sum_qd = 0, sum_d = 0;
    for (int32_t t = e + 1; t < end; ++t) {
        uint64_t c;
        uint32_t d;
        stage_terms(P, u, P.entry_stage[t], A.qlen, A.qdelay, c, d);
        sum_qd += c;
        sum_d += d;
    }
    uint64_t v = sum_qd;                                        // PARD_SUB_LOWER
    if (A.variant == PARD_SUB_UPPER) v = sum_qd + sum_d;
    else if (A.variant == PARD_SUB_SF) v = sum_d;
    if (v > kSubCap) v = kSubCap;
    if (v) atomicMax(&A.sub[(int64_t)u * P.S + k], (unsigned long long)v);
}

// The arrival every (sample, stage) pair draws depends on neither the snapshot nor the path:
// gather them once per call, stage-major, so that the per-path kernel below reads them with
// unit stride instead of chasing two dependent random loads per pair.
__global__ __launch_bounds__(256) void drawn_arrivals_kernel(int32_t S, uint32_t M, const int32_t* samples, const uint32_t* picks,
                                                             uint32_t m_mul, uint32_t m_shf, uint32_t* drawn) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;       // t = j * S + i, the layout of picks
    if (t >= (int64_t)M * S) return;
    const uint32_t pick = picks[t];
    const int32_t a = samples[pick - magic_div_dev(pick, m_mul, m_shf) * M];
    const uint32_t j = (uint32_t)(t / S), i = (uint32_t)(t - (int64_t)j * S);
    drawn[(int64_t)i * M + j] = a > 0 ? (uint32_t)a : 0u;
}

// The sampled variant: one workgroup per (snapshot, path entry).
constexpr int kWThreads = 512;
constexpr int kWWaves = kWThreads / kWave;
constexpr int kWUnroll = 8;                            // samples a thread works on at once
constexpr int kSelBits = 11;                            // radix-select digits: 11 + 11 + 10 bits
constexpr int kSelBins = 1 << kSelBits;

struct WaitLds {
    uint32_t hist[kSelBins];
    uint32_t dur[PARD_MAX_STAGES], mul[PARD_MAX_STAGES], shf[PARD_MAX_STAGES];
    int32_t stg[PARD_MAX_STAGES];
    unsigned long long sum_qd;
    uint32_t sum_d;
    uint32_t wave_tot[kWWaves];
    uint32_t sel_bin, sel_before;
};

__global__ __launch_bounds__(kWThreads) void sub_quantile_kernel(SubArgs A) {
    extern __shared__ __align__(16) uint32_t totals[];          // [num_samples]
    __shared__ WaitLds L;
    const PlanDev& P = A.plan;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int32_t u, e;
    if (!entry_of(P, blockIdx.x, u, e)) return;
    const int32_t k = P.entry_stage[e], end = P.entry_end[e];
    const int len = end - e - 1;                                // stages after k on this path
    if (len <= 0) return;                                       // nothing downstream: 0, the initial value
    const uint32_t M = (uint32_t)A.num_samples;
    if (tid == 0) { L.sum_qd = 0ull; L.sum_d = 0u; }
    __syncthreads();
    if (tid < len) {
        const int32_t i = P.entry_stage[e + 1 + tid];
        uint64_t c;
        uint32_t d;
        stage_terms(P, u, i, A.qlen, A.qdelay, c, d);
        atomicAdd(&L.sum_qd, (unsigned long long)c);
        atomicAdd(&L.sum_d, d);                                 // < 2^32: at most 64 stages of at most 2^25
        // multiply-high constants for x mod d (Granlund & Montgomery, N = 32), d >= 1
        uint32_t mul = 0, shf = 0;
        if (d > 0) {
            const uint32_t l = d > 1 ? 32u - (uint32_t)__clz((int)(d - 1u)) : 0u;      // ceil(log2 d)
            mul = (uint32_t)(wide_div((((uint64_t)1 << l) - d) << 32, d) + 1u);
            shf = (l < 1u ? l : 1u) | ((l > 0u ? l - 1u : 0u) << 8);
        }
        L.dur[tid] = d; L.mul[tid] = mul; L.shf[tid] = shf; L.stg[tid] = i;
    }
    __syncthreads();
    // kWUnroll samples per thread and trip, so that their loads overlap
    for (uint32_t j0 = tid; j0 < M; j0 += kWUnroll * kWThreads) {
        uint32_t total[kWUnroll];
#pragma unroll
        for (int x = 0; x < kWUnroll; ++x) total[x] = 0;
        for (int l = 0; l < len; ++l) {
            const uint32_t d = L.dur[l];
            if (d == 0) continue;
            const uint32_t mul = L.mul[l], shf = L.shf[l];
            const uint32_t* col = A.drawn + (int64_t)L.stg[l] * M;
            uint32_t a[kWUnroll];
#pragma unroll
            for (int x = 0; x < kWUnroll; ++x) {
                const uint32_t j = j0 + x * kWThreads;
                a[x] = col[j < M ? j : j0];
            }
#pragma unroll
            for (int x = 0; x < kWUnroll; ++x) {
                const uint32_t rem = a[x] - magic_div_dev(a[x], mul, shf) * d;
                total[x] += rem ? d - rem : 0u;
            }
        }
#pragma unroll
        for (int x = 0; x < kWUnroll; ++x)
            if (j0 + x * kWThreads < M) totals[j0 + x * kWThreads] = total[x];
    }
    // rank-th smallest total: rounds of counting by 11-bit digit, most significant first.  Every
    // total is below sum d_i, so the digits start at its top bit: the first round then spreads
    // the samples over the counters instead of piling them onto counter 0.
    uint32_t rank = (uint32_t)A.rank, prefix = 0;
    int hi = 32 - __clz((int)(L.sum_d | 1u));                  // bits of the largest possible total
    for (int round = 0; hi > 0; ++round) {
        const int shift = hi > kSelBits ? hi - kSelBits : 0;
        const int bits = hi - shift;
        for (int i = tid; i < kSelBins; i += kWThreads) L.hist[i] = 0;
        __syncthreads();
        for (uint32_t j = tid; j < M; j += kWThreads) {
            const uint32_t v = totals[j];
            if (round == 0 || (v >> (shift + bits)) == prefix) atomicAdd(&L.hist[(v >> shift) & ((1u << bits) - 1u)], 1u);   // round 0: no bits above
        }
        __syncthreads();
        // thread t owns bins 8t..8t+7: find the bin that holds the rank-th candidate
        uint32_t h[kSelBins / kWThreads], mine = 0;
#pragma unroll
        for (int i = 0; i < kSelBins / kWThreads; ++i) { h[i] = L.hist[tid * (kSelBins / kWThreads) + i]; mine += h[i]; }
        uint32_t inc = mine;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t t = __shfl_up(inc, off);
            if (lane >= off) inc += t;
        }
        if (lane == 63) L.wave_tot[wave] = inc;
        __syncthreads();
        uint32_t before = inc - mine;
        for (int w = 0; w < wave; ++w) before += L.wave_tot[w];
        if (rank > before && rank <= before + mine) {            // exactly one thread
            uint32_t run = before;
#pragma unroll
            for (int i = 0; i < kSelBins / kWThreads; ++i) {
                if (rank > run && rank <= run + h[i]) { L.sel_bin = (uint32_t)(tid * (kSelBins / kWThreads) + i); L.sel_before = run; }
                run += h[i];
            }
        }
        __syncthreads();
        prefix = (prefix << bits) | L.sel_bin;
        rank -= L.sel_before;
        hi = shift;
        __syncthreads();
    }
    if (tid == 0) {
        uint64_t v = L.sum_qd + prefix;
        if (v > kSubCap) v = kSubCap;
        if (v) atomicMax(&A.sub[(int64_t)u * P.S + k], (unsigned long long)v);
    }
}

// ---- adaptive priority (Section 3.3) --------------------------------------------------------
// One wave per rate series, 64 samples at a time.  The window sum at t is the prefix sum of
// rate[t] - rate[t - w], so one running scan gives the smoothed workload.  The two thresholds are
// comparisons of rate * lat[B] * sum with a constant of the series, so each is one cut in the
// 32-bit range of a rate: the wave finds both cuts once (six rounds of 64 candidates each, exact
// 128-bit products) and then walks the series backwards (it is in cache) to the last sample that
// lies outside the band - the priority in force at the end, since samples inside change nothing.
constexpr int kPThreads = 256;

__device__ __forceinline__ unsigned __int128 mul_64_64(uint64_t a, uint64_t b) {
    return ((unsigned __int128)__umul64hi(a, b) << 64) | (unsigned __int128)(a * b);
}

// inclusive prefix sum of a 64-bit value across the wave (the 32-bit halves travel separately)
__device__ __forceinline__ int64_t wave_inclusive_sum64(int64_t v) {
    uint64_t x = (uint64_t)v;
#define PARD_SCAN64_STEP(ctrl, rows)                                                                              \
    {                                                                                                             \
        const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)x, ctrl, rows, 0xF, false);   \
        const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(x >> 32), ctrl, rows, 0xF, false); \
        x += ((uint64_t)hi << 32) | lo;                                                                           \
    }
    PARD_SCAN64_STEP(0x111, 0xF)     // row_shr:1
    PARD_SCAN64_STEP(0x112, 0xF)     // row_shr:2
    PARD_SCAN64_STEP(0x114, 0xF)     // row_shr:4
    PARD_SCAN64_STEP(0x118, 0xF)     // row_shr:8
    PARD_SCAN64_STEP(0x142, 0xA)     // row_bcast:15 into rows 1, 3
    PARD_SCAN64_STEP(0x143, 0xC)     // row_bcast:31 into rows 2, 3
#undef PARD_SCAN64_STEP
    return (int64_t)x;
}

// y * d as 128 bits, d given as three 32-bit limbs (d < 2^96), y < 2^32
__device__ __forceinline__ unsigned __int128 mul_32_96(uint32_t y, uint32_t d0, uint32_t d1, uint32_t d2) {
    const uint64_t t0 = (uint64_t)y * d0;
    const uint64_t t1 = (uint64_t)y * d1 + (t0 >> 32);
    const uint64_t t2 = (uint64_t)y * d2 + (t1 >> 32);
    return ((unsigned __int128)t2 << 64) | ((unsigned __int128)(uint32_t)t1 << 32) | (unsigned __int128)(uint32_t)t0;
}

// The number of 32-bit values y, counted from 0 upwards, for which  y * d > bound  (strict) or  y * d >= bound
// (!strict) does NOT hold yet; the condition holds for every y from that number on (2^32 when it never holds).
// All lanes take part and get the same result.
__device__ __forceinline__ uint64_t first_above(uint32_t d0, uint32_t d1, uint32_t d2, unsigned __int128 bound, bool strict, int lane) {
    uint64_t found = 0;                                  // so many values are known not to satisfy the condition
#pragma unroll
    for (int shift = 30; shift >= 0; shift -= 6) {
        const uint64_t y = found + ((uint64_t)(lane + 1) << shift) - 1ull;        // the last of lane+1 more blocks of 2^shift values
        bool short_of = false;
        if (y <= 0xFFFFFFFFull) {
            const unsigned __int128 prod = mul_32_96((uint32_t)y, d0, d1, d2);
            short_of = strict ? !(prod > bound) : !(prod >= bound);
        }
        // the condition is monotone in y, so the lanes that are still short of it form a prefix
        found += (uint64_t)__popcll(__ballot(short_of)) << shift;
    }
    return found;
}

__global__ __launch_bounds__(kPThreads) void priority_modes_kernel(PlanDev P, int32_t T, int32_t window, uint32_t w_mul, uint32_t w_shf,
                                                                   const int32_t* rate, const int32_t* prev_mode, int32_t* mode_out) {
    const int lane = threadIdx.x & 63;
    const int64_t series = (int64_t)P.K * P.S;
    const int64_t wave_id = ((int64_t)blockIdx.x * kPThreads + threadIdx.x) >> 6;
    const int64_t waves = ((int64_t)gridDim.x * kPThreads) >> 6;
    // every series starts on a 16-byte boundary when the array does and the length is a multiple of 4
    const bool vec = (T & 3) == 0 && (reinterpret_cast<uintptr_t>(rate) & 15) == 0;
    for (int64_t g = wave_id; g < series; g += waves) {
        const int64_t rec = P.shared ? g % P.S : g;
        const StageRec sr = P.recs[rec];
        const int32_t* r = rate + g * T;
        // sum of the series and of |rate - smoothed rate|; a lane takes four consecutive samples
        uint64_t sum = 0, dev = 0;
        int64_t carry = 0;                                          // window sum up to the previous chunk's last sample
        for (int32_t t0 = 0; t0 < T; t0 += 4 * 64) {
            const int32_t t = t0 + 4 * lane;
            int32_t xs[4];
            if (vec && t + 3 < T) {
                const int4 v = *reinterpret_cast<const int4*>(r + t);
                xs[0] = v.x; xs[1] = v.y; xs[2] = v.z; xs[3] = v.w;
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) xs[i] = t + i < T ? r[t + i] : 0;
            }
            int64_t part[4];                                         // inc of this lane's samples up to and including i
            int64_t run = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const bool ok = t + i < T;
                const int64_t old = (ok && t + i >= window) ? (int64_t)r[t + i - window] : 0;
                run += (ok ? (int64_t)xs[i] : 0) - old;
                part[i] = run;
            }
            const int64_t incl = wave_inclusive_sum64(run);
            const int64_t before = carry + incl - run;               // window sum just before this lane's first sample
            carry += (int64_t)(((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)((uint64_t)incl >> 32), 63) << 32) |
                               (uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(uint64_t)incl, 63));
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (t + i < T) {
                    const int64_t win = before + part[i];            // rate[max(0, t-w+1)] + ... + rate[t]
                    const int64_t x = (int64_t)xs[i];
                    const int64_t cnt = t + i + 1 < window ? t + i + 1 : window;
                    // floor of the window mean; a sum that fits 32 bits divides by multiplication once the window is
                    // full and by a 32-bit division before that
                    int64_t ts;
                    if (((uint64_t)win >> 32) != 0ull) ts = win / cnt;
                    else if (cnt == window) ts = (int64_t)magic_div_dev((uint32_t)win, w_mul, w_shf);
                    else ts = (int64_t)((uint32_t)win / (uint32_t)cnt);
                    const int64_t d = x - ts;
                    dev += (uint64_t)(d < 0 ? -d : d);
                    sum += (uint64_t)x;
                }
            }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            sum += __shfl_xor(sum, off);
            dev += __shfl_xor(dev, off);
        }
        // thresholds, cross-multiplied:  mu > 1 + eps  <=>  rate * lat[B] * sum > W * B * 10^6 * (sum + dev),
        // mu < 1 - eps  <=>  rate * lat[B] * sum < W * B * 10^6 * (sum - dev); an all-zero series has eps = 0
        const uint64_t cap = (uint64_t)(uint32_t)sr.W * (uint32_t)sr.B * 1000000ull;            // < 2^46
        const uint64_t s1 = sum > 0 ? sum : 1ull, dv = sum > 0 ? dev : 0ull;
        const unsigned __int128 hi = mul_64_64(cap, s1 + dv);
        const bool never_below = dv > s1;                                                         // 1 - eps < 0
        const unsigned __int128 lo = never_below ? (unsigned __int128)0 : mul_64_64(cap, s1 - dv);
        const unsigned __int128 per_rate = mul_64_64((uint64_t)(uint32_t)sr.latB, s1);            // < 2^31 * 2^62
        const uint32_t d0 = (uint32_t)per_rate, d1 = (uint32_t)(per_rate >> 32), d2 = (uint32_t)(per_rate >> 64);
        // a rate is above the band from `above_from` on and below it up to `below_until` - 1
        const uint64_t above_from = first_above(d0, d1, d2, hi, true, lane);
        const uint64_t below_until = never_below ? 0ull : first_above(d0, d1, d2, lo, false, lane);
        int32_t mode = prev_mode ? prev_mode[g] : PARD_ORDER_LBF;
        for (int32_t t0 = ((T - 1) / 64) * 64; t0 >= 0; t0 -= 64) {
            const int32_t t = t0 + lane;
            const bool ok = t < T;
            const uint64_t x = ok ? (uint64_t)(uint32_t)r[t] : 0;
            const bool above = ok && x >= above_from;
            const bool below = ok && x < below_until;
            const unsigned long long decided = __ballot(above || below);
            if (decided) {
                const int last = 63 - __clzll((long long)decided);
                mode = ((__ballot(above) >> last) & 1ull) ? PARD_ORDER_HBF : PARD_ORDER_LBF;
                break;
            }
        }
        if (lane == 0) mode_out[g] = mode;
    }
}

// ---- monitored queueing delay (Section 3.2, State Planner: sliding window over recent delays) ----
// One wave per series of (time, delay) samples.  A sample of age = now - time inside
// [0, window) weighs window - age; the result is floor(sum w * delay / sum w).  Weights and
// delays are below 2^31, so a product fits 62 bits and the sums are carried in 128 bits.
constexpr int kDUnroll = 4;                             // loads of a lane in flight

__global__ __launch_bounds__(kPThreads) void queue_delay_kernel(int32_t K, int32_t S, int32_t len, uint32_t window,
                                                                const int32_t* time, const int32_t* delay,
                                                                const int32_t* now, int32_t* q) {
    const int lane = threadIdx.x & 63;
    const int64_t series = (int64_t)K * S;
    const int64_t wave_id = ((int64_t)blockIdx.x * kPThreads + threadIdx.x) >> 6;
    const int64_t waves = ((int64_t)gridDim.x * kPThreads) >> 6;
    // every series starts on a 16-byte boundary when the arrays do and the length is a multiple of 4
    const bool vec = (len & 3) == 0 && ((reinterpret_cast<uintptr_t>(time) | reinterpret_cast<uintptr_t>(delay)) & 15) == 0;
    for (int64_t g = wave_id; g < series; g += waves) {
        const int64_t t_now = now[g / S];
        const int32_t* tm = time + g * len;
        const int32_t* dl = delay + g * len;
        uint64_t lo = 0, hi = 0, den = 0;
        auto add = [&](bool ok, int32_t t, int32_t x) {
            const int64_t age = t_now - (int64_t)t;
            const bool in = ok && age >= 0 && age < (int64_t)window;
            const uint64_t w = in ? (uint64_t)window - (uint64_t)age : 0ull;
            const uint64_t p = w * (uint64_t)(x > 0 ? (uint32_t)x : 0u);
            lo += p;
            hi += (uint64_t)(lo < p);
            den += w;
        };
        if (vec) {                                      // four samples per load
            const int4* tm4 = reinterpret_cast<const int4*>(tm);
            const int4* dl4 = reinterpret_cast<const int4*>(dl);
            const int32_t len4 = len >> 2;
            for (int32_t j0 = lane; j0 < len4; j0 += 64 * kDUnroll) {
                int4 t[kDUnroll], x[kDUnroll];
#pragma unroll
                for (int i = 0; i < kDUnroll; ++i) {
                    const int32_t j = j0 + 64 * i;
                    const bool ok = j < len4;
                    t[i] = ok ? tm4[j] : make_int4(0, 0, 0, 0);
                    x[i] = ok ? dl4[j] : make_int4(0, 0, 0, 0);
                }
#pragma unroll
                for (int i = 0; i < kDUnroll; ++i) {
                    const bool ok = j0 + 64 * i < len4;
                    add(ok, t[i].x, x[i].x);
                    add(ok, t[i].y, x[i].y);
                    add(ok, t[i].z, x[i].z);
                    add(ok, t[i].w, x[i].w);
                }
            }
        } else {
            for (int32_t j0 = lane; j0 < len; j0 += 64 * kDUnroll) {
                int32_t t[kDUnroll], x[kDUnroll];
#pragma unroll
                for (int i = 0; i < kDUnroll; ++i) {
                    const int32_t j = j0 + 64 * i;
                    const bool ok = j < len;
                    t[i] = ok ? tm[j] : 0;
                    x[i] = ok ? dl[j] : 0;
                }
#pragma unroll
                for (int i = 0; i < kDUnroll; ++i) add(j0 + 64 * i < len, t[i], x[i]);
            }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const uint64_t lo2 = __shfl_xor(lo, off), hi2 = __shfl_xor(hi, off);
            lo += lo2;
            hi += hi2 + (uint64_t)(lo < lo2);
            den += __shfl_xor(den, off);
        }
        if (lane == 0) {
            // the quotient is a weighted mean of values below 2^31: settle its 31 bits from the top
            const unsigned __int128 num = ((unsigned __int128)hi << 64) | (unsigned __int128)lo;
            uint32_t quo = 0;
            if (den > 0)
                for (int b = 30; b >= 0; --b) {
                    const uint32_t cand = quo | (1u << b);
                    if (mul_64_64(den, cand) <= num) quo = cand;
                }
            q[g] = (int32_t)quo;
        }
    }
}

// mode byte of every stage record <- modes[D*S]
__global__ void set_modes_kernel(StageRec* recs, const int32_t* modes, int64_t count) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) recs[i].mode = (recs[i].mode & ~0xFF) | (modes[i] == PARD_ORDER_HBF ? PARD_ORDER_HBF : PARD_ORDER_LBF);
}

}  // namespace

hipError_t launch_priority_modes(const PlanDev& plan, int32_t series_len, int32_t window, const int32_t* rate,
                                 const int32_t* prev_mode, int32_t* mode_out, hipStream_t stream) {
    const int64_t series = (int64_t)plan.K * plan.S;
    int64_t grid = (series + 3) / 4;
    if (grid > 4096) grid = 4096;
    const Magic32 mw = magic_u32((uint32_t)window);
    priority_modes_kernel<<<(unsigned)grid, kPThreads, 0, stream>>>(plan, series_len, window, mw.m, mw.sh, rate, prev_mode, mode_out);
    return hipGetLastError();
}

hipError_t launch_queue_delay(int32_t K, int32_t S, int32_t len, uint32_t window, const int32_t* time, const int32_t* delay,
                              const int32_t* now, int32_t* q, hipStream_t stream) {
    const int64_t series = (int64_t)K * S;
    int64_t grid = (series + 3) / 4;
    if (grid > 8192) grid = 8192;
    queue_delay_kernel<<<(unsigned)grid, kPThreads, 0, stream>>>(K, S, len, window, time, delay, now, q);
    return hipGetLastError();
}

hipError_t launch_set_modes(StageRec* recs, const int32_t* modes, int64_t count, hipStream_t stream) {
    set_modes_kernel<<<(unsigned)((count + 255) / 256), 256, 0, stream>>>(recs, modes, count);
    return hipGetLastError();
}

hipError_t launch_queue_lengths(const PlanDev& plan, int64_t n, const int32_t* stage, const int32_t* snap_ptr,
                                int32_t* qlen, hipStream_t stream) {
    const int64_t segs = (int64_t)plan.K * plan.S;
    int zb = (int)((segs + 255) / 256);
    if (zb > 1024) zb = 1024;
    fill_zero32_kernel<<<zb, 256, 0, stream>>>(qlen, segs);
    if (n > 0) {
        const int64_t grid = (n + kQChunk - 1) / kQChunk;
        queue_lengths_kernel<<<(unsigned)grid, kQThreads, 0, stream>>>(plan.K, plan.S, n, stage, snap_ptr, qlen);
    }
    return hipGetLastError();
}

hipError_t launch_sub_latency(const SubArgs& a, hipStream_t stream) {
    const PlanDev& P = a.plan;
    const int64_t segs = (int64_t)P.K * P.S;
    int zb = (int)((segs + 255) / 256);
    if (zb > 1024) zb = 1024;
    fill_zero_kernel<<<zb, 256, 0, stream>>>(a.sub, segs);
    if (a.variant == PARD_SUB_BACK) return hipGetLastError();
    const int64_t items = P.shared ? (int64_t)P.K * P.max_entries_per_dag : P.total_entries;
    if (items <= 0) return hipGetLastError();
    if (a.variant != PARD_SUB_FULL) {
        sub_simple_kernel<<<(unsigned)((items + 255) / 256), 256, 0, stream>>>(a, items);
    } else {
        const Magic32 mm = magic_u32((uint32_t)a.num_samples);
        const int64_t pairs = (int64_t)a.num_samples * P.S;
        drawn_arrivals_kernel<<<(unsigned)((pairs + 255) / 256), 256, 0, stream>>>(P.S, (uint32_t)a.num_samples, a.samples, a.picks,
                                                                                  mm.m, mm.sh, a.drawn);
        sub_quantile_kernel<<<(unsigned)items, kWThreads, (size_t)a.num_samples * 4, stream>>>(a);
    }
    return hipGetLastError();
}

}  // namespace pard
