// Out-of-core path for snapshots larger than one workgroup's on-chip capacity.
//
// Steps (paper Section 3.2 Eq.(1),(2),(4), DAG maximum; Section 3.3 ordering):
//   count     per-(snapshot, stage) queue lengths and the key range
//   setup     queue offsets (exclusive scan), cost of every stage at its full queue
//             length, downstream maximum per (snapshot, stage) over the path CSR
//   histogram digit histograms of every radix pass in one read of the input
//   passes    stable least-significant-digit radix sort of (segment, key) with 8-bit
//             digits; one kernel per digit, each tile's global offsets obtained by a
//             decoupled look-back over the tiles before it (single read + single write
//             of the data per pass)
//   epilogue  queue position = sorted position - queue offset; own-stage cost +
//             downstream maximum; drop decision; est/drop scattered to request order.
//
// The sort key is the virtual integer  V = segment << kb | (key - min key)  where kb is
// the number of bits of the key range; only ceil(bits(V)/8) passes run.  The segment id
// travels in the otherwise unused top bits of the 32-bit request index.
#include "pard_device.hpp"

namespace pard {

namespace {

constexpr int kRadixBits = 8;
constexpr int kRadix = 1 << kRadixBits;
constexpr int kSortThreads = 256;
constexpr int kSortItems = 16;
constexpr int kTile = kSortThreads * kSortItems;       // 4096 elements per tile
constexpr int kSortWaves = kSortThreads / kWave;
constexpr int kMaxPasses = 8;
constexpr uint32_t kFlagAggregate = 1u << 30;          // tile published its own count
constexpr uint32_t kFlagInclusive = 2u << 30;          // tile published the running total
constexpr uint32_t kValueMask = (1u << 30) - 1;
constexpr uint32_t kSpinLimit = 1u << 22;

struct SortParams {                 // lives in device memory, written by the setup kernel
    uint32_t inv_min;               // max over requests of ~key  (so that zero-fill is the identity)
    uint32_t max_key;
    uint32_t kb;                    // bits of (max key - min key)
    uint32_t passes;                // radix passes actually needed
    uint32_t ticket[kMaxPasses];    // next tile number of each pass
};

struct SortLayout {
    int64_t params, seg_count, cfull, down, hist, status, zero_end, key[2], pay[2], total;
    int64_t tiles;
    int32_t max_passes, idx_bits, seg_bits;
};

int bits_of(uint64_t x) { int b = 0; while (x) { ++b; x >>= 1; } return b; }
int64_t align256(int64_t x) { return (x + 255) & ~(int64_t)255; }

SortLayout make_layout(int32_t K, int32_t S, int64_t n) {
    SortLayout L{};
    const int64_t segs = (int64_t)K * S;
    L.idx_bits = bits_of(n > 0 ? (uint64_t)(n - 1) : 0);
    L.seg_bits = bits_of((uint64_t)(segs - 1));
    L.max_passes = (32 + L.seg_bits + kRadixBits - 1) / kRadixBits;
    L.tiles = (n + kTile - 1) / kTile;
    int64_t off = 0;
    L.params = off;     off = align256(off + (int64_t)sizeof(SortParams));
    L.seg_count = off;  off = align256(off + segs * 4);
    L.cfull = off;      off = align256(off + segs * 8);
    L.down = off;       off = align256(off + segs * 8);
    L.hist = off;       off = align256(off + (int64_t)kMaxPasses * kRadix * 4);
    L.status = off;     off = align256(off + (int64_t)L.max_passes * L.tiles * kRadix * 4);
    L.zero_end = off;
    for (int b = 0; b < 2; ++b) {
        L.key[b] = off; off = align256(off + n * 4);
        L.pay[b] = off; off = align256(off + n * 4);
    }
    L.total = off;
    return L;
}

struct SortDev {                    // everything the sort kernels need, by value
    PlanDev plan;
    int64_t n;
    const int32_t *arrival, *deadline, *stage, *snap_ptr, *now;
    int32_t* est;
    uint8_t* drop;
    int32_t *order, *seg_ptr;
    uint32_t* status_word;
    SortParams* params;
    uint32_t* seg_count;
    unsigned long long *cfull, *down;
    uint32_t* hist;                 // [kMaxPasses][256]
    uint32_t* tile_status;          // [max_passes][tiles][256]
    uint32_t* key[2];
    uint32_t* pay[2];
    int64_t tiles;
    int32_t idx_bits, seg_bits, max_passes;
};

__global__ void zero_kernel(uint4* p, int64_t count16) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < count16; i += stride) p[i] = make_uint4(0, 0, 0, 0);
}

// snapshot of request r: the u with snap_ptr[u] <= r < snap_ptr[u+1]
__device__ __forceinline__ int32_t snapshot_of(const int32_t* snap_ptr, int32_t K, int64_t r) {
    if (K == 1) return 0;
    int32_t lo = 0, hi = K;                       // first u in (lo, hi] with snap_ptr[u] > r
    while (hi - lo > 1) {
        int32_t mid = (lo + hi) >> 1;
        if ((int64_t)snap_ptr[mid] <= r) lo = mid; else hi = mid;
    }
    return lo;
}

__device__ __forceinline__ void request_segment_key(const SortDev& A, int64_t r, uint32_t& seg, uint32_t& key) {
    const PlanDev& P = A.plan;
    const int32_t u = snapshot_of(A.snap_ptr, P.K, r);
    const int32_t s = clamp_stage(A.stage[r], P.S);
    const int32_t mode = P.uniform_mode >= 0 ? P.uniform_mode
                                             : P.recs[(P.shared ? 0 : (int64_t)u * P.S) + s].mode;
    const int32_t arr = (P.any_fcfs && mode == PARD_ORDER_FCFS) ? A.arrival[r] : 0;
    seg = (uint32_t)u * (uint32_t)P.S + (uint32_t)s;
    key = order_key(mode, A.deadline[r], arr);
}

// ---- count: queue lengths and key range ------------------------------------------
constexpr int kCountLds = 4096;
__global__ __launch_bounds__(256) void count_kernel(SortDev A) {
    __shared__ uint32_t h[kCountLds];
    const int64_t segs = (int64_t)A.plan.K * A.plan.S;
    const bool use_lds = segs <= kCountLds;            // privatise the counters when they fit
    if (use_lds) {
        for (int i = threadIdx.x; i < segs; i += 256) h[i] = 0;
        __syncthreads();
    }
    uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < A.n; r += stride) {
        uint32_t seg, key;
        request_segment_key(A, r, seg, key);
        if (use_lds) atomicAdd(&h[seg], 1u); else atomicAdd(&A.seg_count[seg], 1u);
        kmin = key < kmin ? key : kmin;
        kmax = key > kmax ? key : kmax;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        uint32_t a = __shfl_xor(kmin, off), b = __shfl_xor(kmax, off);
        kmin = a < kmin ? a : kmin;
        kmax = b > kmax ? b : kmax;
    }
    if ((threadIdx.x & (kWave - 1)) == 0) {
        atomicMax(&A.params->inv_min, ~kmin);
        atomicMax(&A.params->max_key, kmax);
    }
    if (use_lds) {
        __syncthreads();
        for (int i = threadIdx.x; i < segs; i += 256)
            if (h[i]) atomicAdd(&A.seg_count[i], h[i]);
    }
}

// ---- setup: one workgroup --------------------------------------------------------
__global__ __launch_bounds__(1024) void setup_kernel(SortDev A) {
    __shared__ uint32_t wave_tot[16];
    __shared__ uint32_t carry;
    const PlanDev& P = A.plan;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t segs = (int64_t)P.K * P.S;
    if (tid == 0) {
        const uint32_t umin = ~A.params->inv_min;
        const uint32_t range = A.n > 0 ? A.params->max_key - umin : 0u;
        const uint32_t kb = 32u - (range ? (uint32_t)__clz((int)range) : 32u);
        const uint32_t total = kb + (uint32_t)A.seg_bits;
        uint32_t passes = (total + kRadixBits - 1) / kRadixBits;
        A.params->kb = kb;
        A.params->passes = passes < 1 ? 1 : passes;
        carry = 0;
    }
    __syncthreads();
    // queue offsets: exclusive scan of the queue lengths, 1024 at a time
    for (int64_t base = 0; base < segs + 1; base += 1024) {
        const int64_t g = base + tid;
        const uint32_t v = g < segs ? A.seg_count[g] : 0u;
        uint32_t inc = v;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            uint32_t t = __shfl_up(inc, off);
            if (lane >= off) inc += t;
        }
        if (lane == 63) wave_tot[wave] = inc;
        __syncthreads();
        uint32_t pre = carry;
        for (int w = 0; w < wave; ++w) pre += wave_tot[w];
        if (g <= segs) A.seg_ptr[g] = (int32_t)(pre + inc - v);
        __syncthreads();
        if (tid == 1023) carry = pre + inc;
        __syncthreads();
    }
    // cost of every stage at its full queue length
    for (int64_t g = tid; g < segs; g += 1024) {
        const int64_t rec = P.shared ? g % P.S : g;
        A.cfull[g] = stage_cost(P.recs[rec], A.seg_count[g], P.lat + rec * PARD_LAT_ENTRIES);
    }
    __threadfence_block();
    __syncthreads();
    // downstream maximum per (snapshot, stage): suffix sums along every path
    for (int32_t u = 0; u < P.K; ++u) {
        const int32_t dag = P.shared ? 0 : u;
        const int32_t e_lo = P.dag_entry_ptr[dag], e_hi = P.dag_entry_ptr[dag + 1];
        for (int32_t e = e_lo + tid; e < e_hi; e += 1024) {
            const int32_t end = P.entry_end[e];
            unsigned long long sum = 0;
            for (int32_t t = e + 1; t < end; ++t) sum += A.cfull[(int64_t)u * P.S + P.entry_stage[t]];
            atomicMax(&A.down[(int64_t)u * P.S + P.entry_stage[e]], sum);
        }
    }
}

__device__ __forceinline__ uint32_t digit_of(uint32_t key, uint32_t seg, uint32_t kb, int pass) {
    const uint64_t v = ((uint64_t)seg << kb) | (uint64_t)key;
    return (uint32_t)(v >> (kRadixBits * pass)) & (kRadix - 1);
}

// ---- histogram of every pass's digit -------------------------------------------------
__global__ __launch_bounds__(256) void histogram_kernel(SortDev A) {
    __shared__ uint32_t h[kMaxPasses * kRadix];
    const int tid = threadIdx.x;
    for (int i = tid; i < kMaxPasses * kRadix; i += 256) h[i] = 0;
    __syncthreads();
    const uint32_t umin = ~A.params->inv_min, kb = A.params->kb;
    const int passes = (int)A.params->passes;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t r = (int64_t)blockIdx.x * blockDim.x + tid; r < A.n; r += stride) {
        uint32_t seg, key;
        request_segment_key(A, r, seg, key);
        key -= umin;
        for (int p = 0; p < passes; ++p) atomicAdd(&h[p * kRadix + digit_of(key, seg, kb, p)], 1u);
    }
    __syncthreads();
    for (int i = tid; i < passes * kRadix; i += 256)
        if (h[i]) atomicAdd(&A.hist[i], h[i]);
}

// exclusive scan of one value per thread over a 256-thread workgroup
__device__ __forceinline__ uint32_t block_exclusive_scan_256(uint32_t v, uint32_t* tmp /*[4]*/, int tid) {
    const int lane = tid & 63, wave = tid >> 6;
    uint32_t inc = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        uint32_t t = __shfl_up(inc, off);
        if (lane >= off) inc += t;
    }
    __syncthreads();                    // tmp may still be read from a previous call
    if (lane == 63) tmp[wave] = inc;
    __syncthreads();
    uint32_t pre = 0;
    for (int w = 0; w < wave; ++w) pre += tmp[w];
    return pre + inc - v;
}

// ---- one radix pass --------------------------------------------------------------------
template <bool FIRST>
__global__ __launch_bounds__(kSortThreads) void sort_pass_kernel(SortDev A, int pass) {
    if (pass >= (int)A.params->passes) return;

    __shared__ uint32_t lds_key[kTile];
    __shared__ uint32_t lds_pay[kTile];
    __shared__ uint32_t whist[kSortWaves][kRadix];
    __shared__ uint32_t tile_start[kRadix];
    __shared__ uint32_t gbase[kRadix];
    __shared__ uint32_t scan_tmp[kSortWaves];
    __shared__ uint32_t s_tile;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) s_tile = atomicAdd(&A.params->ticket[pass], 1u);
    for (int i = tid; i < kSortWaves * kRadix; i += kSortThreads) (&whist[0][0])[i] = 0;
    __syncthreads();
    const int64_t tile = s_tile;
    if (tile >= A.tiles) return;                       // cannot happen: one ticket per workgroup
    const int64_t tile_base = tile * kTile;
    const int valid = (int)((A.n - tile_base) < kTile ? (A.n - tile_base) : kTile);
    const uint32_t umin = ~A.params->inv_min, kb = A.params->kb;
    const uint32_t* src_key = A.key[(pass + 1) & 1];
    const uint32_t* src_pay = A.pay[(pass + 1) & 1];
    uint32_t* dst_key = A.key[pass & 1];
    uint32_t* dst_pay = A.pay[pass & 1];

    // load (wave-striped: wave w owns elements [w*1024, (w+1)*1024) of the tile, item i lane l
    // is element w*1024 + i*64 + l), rank every element among equal digits before it
    uint32_t key[kSortItems], pay[kSortItems], rd[kSortItems];   // rd = rank | digit << 16
#pragma unroll
    for (int i = 0; i < kSortItems; ++i) {
        const int e = wave * (kWave * kSortItems) + i * kWave + lane;
        const bool ok = e < valid;
        key[i] = 0;
        pay[i] = 0;
        if (ok) {
            if (FIRST) {
                uint32_t seg, k;
                request_segment_key(A, tile_base + e, seg, k);
                key[i] = k - umin;
                pay[i] = (uint32_t)(tile_base + e) | (seg << A.idx_bits);
            } else {
                key[i] = src_key[tile_base + e];
                pay[i] = src_pay[tile_base + e];
            }
        }
    }
#pragma unroll
    for (int i = 0; i < kSortItems; ++i) {
        const int e = wave * (kWave * kSortItems) + i * kWave + lane;
        const bool ok = e < valid;
        const uint32_t d = digit_of(key[i], A.idx_bits < 32 ? (pay[i] >> A.idx_bits) : 0u, kb, pass);
        unsigned long long peers = __ballot(ok);
#pragma unroll
        for (int b = 0; b < kRadixBits; ++b) {
            const bool bit = (d >> b) & 1u;
            const unsigned long long vote = __ballot(bit);
            peers &= bit ? vote : ~vote;
        }
        const uint32_t before = __builtin_amdgcn_mbcnt_hi((uint32_t)(peers >> 32),
                                    __builtin_amdgcn_mbcnt_lo((uint32_t)peers, 0u));
        const uint32_t count = (uint32_t)__popcll(peers);
        uint32_t prev = 0;
        if (ok) {
            prev = whist[wave][d];
            if (before == count - 1) whist[wave][d] = prev + count;   // last peer advances the counter
        }
        rd[i] = (prev + before) | (d << 16);
    }
    __syncthreads();

    // per digit: offsets of each wave's run inside the tile, tile count, global offset
    {
        const int d = tid;                                   // kSortThreads == kRadix
        uint32_t run = 0;
#pragma unroll
        for (int w = 0; w < kSortWaves; ++w) {
            const uint32_t t = whist[w][d];
            whist[w][d] = run;
            run += t;
        }
        const uint32_t tile_cnt = run;
        uint32_t* st = A.tile_status + ((int64_t)pass * A.tiles + tile) * kRadix + d;
        if (tile == 0)
            __hip_atomic_store(st, kFlagInclusive | tile_cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else
            __hip_atomic_store(st, kFlagAggregate | tile_cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const uint32_t bin_base = block_exclusive_scan_256(A.hist[pass * kRadix + d], scan_tmp, tid);
        const uint32_t tstart = block_exclusive_scan_256(tile_cnt, scan_tmp, tid);
        tile_start[d] = tstart;
        uint32_t excl = 0;
        if (tile > 0) {
            int64_t t = tile - 1;
            uint32_t spins = 0;
            while (true) {
                const uint32_t v = __hip_atomic_load(A.tile_status + ((int64_t)pass * A.tiles + t) * kRadix + d,
                                                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const uint32_t flag = v & ~kValueMask;
                if (flag == 0) {
                    if (++spins > kSpinLimit) { atomicOr(A.status_word, kStatusLookbackTimeout); break; }
                    __builtin_amdgcn_s_sleep(2);
                    continue;
                }
                excl += v & kValueMask;
                if (flag == kFlagInclusive) break;
                --t;                                          // tile 0 always publishes inclusive
            }
            __hip_atomic_store(st, kFlagInclusive | ((excl + tile_cnt) & kValueMask),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        gbase[d] = bin_base + excl - tstart;
    }
    __syncthreads();

    // reorder inside the tile so that equal digits are contiguous, then write runs out
#pragma unroll
    for (int i = 0; i < kSortItems; ++i) {
        const int e = wave * (kWave * kSortItems) + i * kWave + lane;
        if (e < valid) {
            const uint32_t d = rd[i] >> 16;
            const uint32_t lp = tile_start[d] + whist[wave][d] + (rd[i] & 0xFFFFu);
            lds_key[lp] = key[i];
            lds_pay[lp] = pay[i];
        }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kSortItems; ++i) {
        const int j = i * kSortThreads + tid;
        if (j < valid) {
            const uint32_t k = lds_key[j], p = lds_pay[j];
            const uint32_t d = digit_of(k, A.idx_bits < 32 ? (p >> A.idx_bits) : 0u, kb, pass);
            const uint32_t dst = gbase[d] + (uint32_t)j;
            if ((int64_t)dst < A.n) { dst_key[dst] = k; dst_pay[dst] = p; }
        }
    }
}

// ---- epilogue: positions -> estimates, drop decisions, queue order ------------------------
__global__ __launch_bounds__(256) void epilogue_kernel(SortDev A) {
    const PlanDev& P = A.plan;
    const int last = ((int)A.params->passes - 1) & 1;
    const uint32_t* keys = A.key[last];
    const uint32_t* pays = A.pay[last];
    const uint32_t umin = ~A.params->inv_min;
    const uint32_t idx_mask = A.idx_bits >= 32 ? 0xFFFFFFFFu : ((1u << A.idx_bits) - 1u);
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < A.n; j += stride) {
        const uint32_t p = pays[j];
        const uint32_t r = p & idx_mask;
        const uint32_t seg = A.idx_bits < 32 ? (p >> A.idx_bits) : 0u;
        const uint32_t u = seg / (uint32_t)P.S, k = seg - u * (uint32_t)P.S;
        const int64_t rec = P.shared ? (int64_t)k : (int64_t)seg;
        const StageRec sr = P.recs[rec];
        const uint32_t pos = (uint32_t)(j - (int64_t)A.seg_ptr[seg]);
        const uint64_t e64 = stage_cost(sr, pos, P.lat + rec * PARD_LAT_ENTRIES) + A.down[seg];
        int32_t deadline;
        const uint32_t uk = keys[j] + umin;
        if (sr.mode == PARD_ORDER_LBF) deadline = (int32_t)(uk ^ 0x80000000u);
        else if (sr.mode == PARD_ORDER_HBF) deadline = (int32_t)(~uk ^ 0x80000000u);
        else deadline = A.deadline[r];
        int32_t est;
        uint8_t drp;
        finish_request(e64, A.now[u], deadline, est, drp);
        A.order[j] = (int32_t)r;
        A.est[r] = est;
        A.drop[r] = drp;
    }
}

SortDev make_dev(const SortArgs& a, const SortLayout& L) {
    SortDev D{};
    char* ws = static_cast<char*>(a.workspace);
    D.plan = a.plan;
    D.n = a.n;
    D.arrival = a.arrival; D.deadline = a.deadline; D.stage = a.stage;
    D.snap_ptr = a.snap_ptr; D.now = a.now;
    D.est = a.est; D.drop = a.drop; D.order = a.order; D.seg_ptr = a.seg_ptr;
    D.status_word = a.status;
    D.params = reinterpret_cast<SortParams*>(ws + L.params);
    D.seg_count = reinterpret_cast<uint32_t*>(ws + L.seg_count);
    D.cfull = reinterpret_cast<unsigned long long*>(ws + L.cfull);
    D.down = reinterpret_cast<unsigned long long*>(ws + L.down);
    D.hist = reinterpret_cast<uint32_t*>(ws + L.hist);
    D.tile_status = reinterpret_cast<uint32_t*>(ws + L.status);
    for (int b = 0; b < 2; ++b) {
        D.key[b] = reinterpret_cast<uint32_t*>(ws + L.key[b]);
        D.pay[b] = reinterpret_cast<uint32_t*>(ws + L.pay[b]);
    }
    D.tiles = L.tiles;
    D.idx_bits = L.idx_bits;
    D.seg_bits = L.seg_bits;
    D.max_passes = L.max_passes;
    return D;
}

}  // namespace

int64_t sort_workspace_bytes(int32_t K, int32_t S, int64_t n) { return make_layout(K, S, n).total; }

bool sort_supported(int32_t K, int32_t S, int64_t n) {
    const SortLayout L = make_layout(K, S, n);
    return L.idx_bits + L.seg_bits <= 32 && n < ((int64_t)1 << 30);
}

hipError_t launch_sort_path(const SortArgs& a, hipStream_t stream) {
    const SortLayout L = make_layout(a.plan.K, a.plan.S, a.n);
    const SortDev D = make_dev(a, L);
    const int64_t zero16 = L.zero_end / 16;
    int zb = (int)((zero16 + 255) / 256);
    if (zb > 4096) zb = 4096;
    if (zb < 1) zb = 1;
    zero_kernel<<<zb, 256, 0, stream>>>(reinterpret_cast<uint4*>(a.workspace), zero16);
    int gb = (int)((a.n + 256 * 8 - 1) / (256 * 8));
    if (gb > 8192) gb = 8192;
    if (gb < 1) gb = 1;
    count_kernel<<<gb, 256, 0, stream>>>(D);
    setup_kernel<<<1, 1024, 0, stream>>>(D);
    if (a.n > 0) {
        histogram_kernel<<<gb, 256, 0, stream>>>(D);
        for (int p = 0; p < L.max_passes; ++p) {
            if (p == 0) sort_pass_kernel<true><<<(unsigned)L.tiles, kSortThreads, 0, stream>>>(D, p);
            else sort_pass_kernel<false><<<(unsigned)L.tiles, kSortThreads, 0, stream>>>(D, p);
        }
        epilogue_kernel<<<gb, 256, 0, stream>>>(D);
    }
    return hipGetLastError();
}

}  // namespace pard
