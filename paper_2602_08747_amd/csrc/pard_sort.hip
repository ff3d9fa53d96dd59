// Out-of-core path for snapshots larger than one workgroup's on-chip capacity.
//
// Steps (paper Section 3.2 Eq.(1),(2),(4), DAG maximum; Section 3.3 ordering):
//   count     per-(snapshot, stage) queue lengths and the key range
//   setup     queue offsets (exclusive scan), cost of every stage at its full queue
//             length, downstream maximum per (snapshot, stage) over the path CSR
//   passes    stable least-significant-digit radix sort of (segment, key) with 8-bit
//             digits.  Per digit: an upsweep reads the keys and leaves every tile's digit
//             histogram, two small kernels turn the histograms into each tile's first
//             output slot per digit (scan over tiles, then over digits), and a downsweep
//             reads the tile again, ranks it and writes it out.  No workgroup waits for
//             another one (a decoupled look-back over ~2000 co-resident tiles cost more
//             than the second read of the keys)
//   results   queue position = sorted position - queue offset; own-stage cost + downstream maximum; drop
//             decision.  Formed inside the last pass (which then writes the queue order instead of its keys)
//             and brought back to request order in two steps: gathered by range of request ids, then one
//             workgroup per range.  Beyond 2^25 requests: est|drop scattered to request order as one word by
//             a kernel of its own, then unpacked by a streaming kernel.
//
// The sort key is the virtual integer  V = segment << kb | (key - min key)  where kb is
// the number of bits of the key range; only ceil(bits(V)/8) passes run.  The payload word
// carries the request's index inside its snapshot (as many bits as the promised snapshot
// bound needs) and the segment id above it; the epilogue adds the snapshot's first request.
#include "pard_device.hpp"
#include <type_traits>

namespace pard {

namespace {

constexpr int kRadixBits = 8;
constexpr int kRadix = 1 << kRadixBits;
constexpr int kSortThreads = 512;
constexpr int kSortItems = 8;                          // elements per thread of a radix pass: a tile holds 4096 elements (three
                                                       // workgroups per compute unit; with 8192, two fit: first downsweep 91 -> 72 us
                                                       // on 16.8 million requests, the call 0.574 -> 0.562 ms),
constexpr int kSmallItems = 4;                         // or 2048 when there are few requests: more, shorter-lived workgroups
                                                       // (a million shuffled requests: 0.171 -> 0.133 ms per call)
constexpr int64_t kSmallTileMax = (int64_t)1 << 22;    // up to this many requests the small tile is used
constexpr int kSortWaves = kSortThreads / kWave;
constexpr int kDies = 8;                               // accelerator dies (XCDs), each with its own L2
constexpr int kChunkTiles = 32;                        // tiles per chunk of the two-level scan over tiles
constexpr int kConsTile = 256;                         // queue slots per workgroup in the consistent-dropping kernels
constexpr int kConsRanges = 8192;                      // workgroups of those kernels at most (each owns a range of tiles)
constexpr int kFusedScanChunks = 128;                  // up to here every chunk scans the chunk totals itself

constexpr int kRetBuckets = 1024;                      // ranges of request ids the results are first gathered by, at most
                                                       // (up to 512 as long as ranges of 2^15 ids cover the requests)
constexpr int kRetMaxShift = 15;                       // a range holds at most 2^15 request ids: its packed results fit one workgroup's LDS
constexpr int kRetMinShift = 11;                       // and at least 2^11 (few requests: more, smaller ranges keep the chip busy)

constexpr uint32_t kSegScan = 1u << 31;                // queue flag: consistent positions by prefix minimum (see below)

struct SortParams {                 // lives in device memory, written by the setup kernel
    uint32_t inv_min;               // max over requests of ~key  (so that zero-fill is the identity)
    uint32_t max_key;
    uint32_t kb;                    // bits of (max key - min key)
    uint32_t passes;                // radix passes actually needed
    uint32_t total_bits;            // bits of the virtual sort key
    uint32_t split;                 // the requests come in deadline order: the queues are a stable split by stage (no sort)
    uint32_t presplit;              // the same under sequentially consistent dropping: the split leaves the sorted keys and
                                    // payloads where the radix passes would have, and the consistent_* kernels go on from there
};

constexpr int kStreamBlocksMax = 1024;                 // upper bound on the grid of the streaming kernels
constexpr int kPartialSegs = 64;                       // up to this many queues: per-workgroup partial counts

struct SortLayout {
    int64_t params, seg_count, cfull, down, keepm, chunk_tot, ret_cursor, zero_end, zero_end_consistent, tile_hist, part_minmax, part_cnt, part_flag, wave_cnt, key[2], pay[2],
            min_lat, alive, wkept, tile_tot, range_tot, carry, total;
    int64_t tiles, chunks;
    int32_t max_passes, idx_bits, seg_bits, ret_shift, tile_items;
};

int bits_of(uint64_t x) { int b = 0; while (x) { ++b; x >>= 1; } return b; }
int64_t align256(int64_t x) { return (x + 255) & ~(int64_t)255; }

SortLayout make_layout(int32_t K, int32_t S, int64_t n, int64_t max_snap) {
    SortLayout L{};
    const int64_t segs = (int64_t)K * S;
    const int64_t span = max_snap < n ? max_snap : n;            // no snapshot holds more requests than this
    L.idx_bits = bits_of(span > 0 ? (uint64_t)(span - 1) : 0);
    L.seg_bits = bits_of((uint64_t)(segs - 1));
    L.max_passes = (32 + L.seg_bits + kRadixBits - 1) / kRadixBits;
    L.ret_shift = bits_of(n > 0 ? (uint64_t)(n - 1) : 0) - 9;       // 512 ranges of 2^ret_shift request ids cover n;
    if (L.ret_shift < kRetMinShift) L.ret_shift = kRetMinShift;
    if (L.ret_shift == kRetMaxShift + 1) L.ret_shift = kRetMaxShift; // up to 2^25 requests: kRetBuckets ranges of the largest size
                                                                    // (beyond that the results go back one by one)
    L.tile_items = n <= kSmallTileMax ? kSmallItems : kSortItems;
    const int64_t tile = (int64_t)kSortThreads * L.tile_items;
    L.tiles = (n + tile - 1) / tile;
    L.chunks = (L.tiles + kChunkTiles - 1) / kChunkTiles;
    int64_t off = 0;
    L.params = off;     off = align256(off + (int64_t)sizeof(SortParams));
    L.seg_count = off;  off = align256(off + segs * 4);
    L.cfull = off;      off = align256(off + segs * 8);
    L.down = off;       off = align256(off + segs * 8);
    const int64_t words = (n + 63) / 64 + 1;                     // 64 queue slots per mask word
    L.chunk_tot = off;  off = align256(off + (int64_t)L.max_passes * L.chunks * kRadix * 4);
    L.ret_cursor = off; off = align256(off + (int64_t)kRetBuckets * 4);
    L.zero_end = off;                                            // zeroed by every call up to here,
    L.keepm = off;      off = align256(off + words * 8);
    L.zero_end_consistent = off;                                 // up to here under sequentially consistent dropping
    L.tile_hist = off;  off = align256(off + (int64_t)L.max_passes * L.tiles * kRadix * 4);
    L.part_minmax = off; off = align256(off + (int64_t)kStreamBlocksMax * 8);
    L.part_cnt = off;    off = align256(off + (int64_t)kStreamBlocksMax * kPartialSegs * 4);
    L.part_flag = off;   off = align256(off + (int64_t)kStreamBlocksMax * 4);
    L.wave_cnt = off;    off = align256(off + (int64_t)kStreamBlocksMax * 16 * kPartialSegs * 4);
    for (int b = 0; b < 2; ++b) {
        L.key[b] = off; off = align256(off + n * 4);
        L.pay[b] = off; off = align256(off + n * 4);
    }
    L.min_lat = off;    off = align256(off + segs * 4);
    L.alive = off;      off = align256(off + words * 8);
    L.wkept = off;      off = align256(off + words * 4);
    const int64_t ctiles = (n + kConsTile - 1) / kConsTile + 1;
    L.tile_tot = off;   off = align256(off + ctiles * 8);
    L.range_tot = off;  off = align256(off + (int64_t)kConsRanges * 8);
    L.carry = off;      off = align256(off + (int64_t)kConsRanges * 4);
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
    const int64_t* sub;
    uint32_t* status_word;
    SortParams* params;
    uint32_t* seg_count;
    unsigned long long *cfull, *down;
    uint32_t* chunk_tot;            // [max_passes][chunks][256] digit counts per chunk of tiles, then their scan
    uint32_t* tile_hist;            // [max_passes][tiles][256] digit counts per tile, then each tile's first output slots
    int64_t chunks;
    uint32_t* part_minmax;          // [stream_blocks][2]  per-workgroup (~min key, max key)
    uint32_t* part_cnt;             // [stream_blocks][kPartialSegs] per-workgroup queue lengths (then, for the split, the
                                    // queue lengths of all workgroups before)
    uint32_t* part_flag;            // [stream_blocks] what a workgroup saw of the order of the deadlines (kSaw*)
    uint32_t* wave_cnt;             // [stream_blocks][16][kPartialSegs] queue lengths of every wave's stretch of the array
    int32_t stream_blocks;
    uint32_t* key[2];
    uint32_t* pay[2];
    int64_t tiles;
    int32_t idx_bits, seg_bits, max_passes;
    uint32_t* ret_cursor;           // [kRetBuckets] results gathered so far per range of request ids (zeroed with the counters)
    int32_t ret_shift;              // a range holds 2^ret_shift request ids
    int32_t finish_in_last_pass;    // the last radix pass forms the results and hands them on by range (epilogue_return_kernel finishes)
    // sequentially consistent dropping
    uint32_t* min_lat;              // [K*S] smallest execution latency a request of the queue can see
    unsigned long long* alive;      // bit j: the request in queue slot j survives at the smallest possible cost
    unsigned long long* keepm;      // bit j: the request in queue slot j is kept (zeroed with the counters)
    uint32_t* wkept;                // [word w]: kept requests of the queue that owns slot 64w, in its slots before 64w
    uint2* tile_tot;                // [tile of kConsTile slots]: (a queue starts, minimum since the last start) over the
                                    // slots before the tile inside its workgroup's range of tiles
    uint2* range_tot;               // [range]: the same pair over the whole range
    int32_t* carry;                 // [range]: minimum over the slots before the range since the last queue start
    int32_t cons_ranges;            // ranges (= workgroups of the prepare and finish kernels)
    int32_t consistent;             // sequentially consistent dropping asked for
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

// the same among the snapshots lo..hi (r is known to lie in one of them)
__device__ __forceinline__ int32_t snapshot_between(const int32_t* snap_ptr, int32_t lo, int32_t hi, int64_t r) {
    int32_t a = lo, b = hi + 1;                   // answer in [a, b)
    while (b - a > 1) {
        const int32_t mid = (a + b) >> 1;
        if ((int64_t)snap_ptr[mid] <= r) a = mid; else b = mid;
    }
    return a;
}

// ---- streaming reads shared by the count and histogram kernels -------------------------
constexpr int kScanThreads = 1024;
constexpr int kScanItems = 8;                          // requests per thread per chunk
constexpr int kChunk = kScanThreads * kScanItems;      // 8192 requests per chunk

// A wave walks a contiguous stretch of the request array kWaveChunk requests at a time: two groups of 256, in each
// of which a lane holds four consecutive requests, so that a load or store of the wave covers whole cache lines
// (16 bytes per lane when the arrays allow it; with eight consecutive requests per lane every access touched
// twice the lines and the two kernels below ran 15 % slower).  Order inside a chunk: group, lane, the four.
constexpr int kWaveChunk = kWave * kScanItems;         // 512 requests
constexpr int kGroupSpan = kWave * 4;                  // 256 requests

// first request of the g-th group of four of a lane
__device__ __forceinline__ int64_t lane_first(int64_t base, int lane, int g) { return base + g * kGroupSpan + lane * 4; }

// The wave chunks [first, last) of wave `wave` of workgroup `block`: the workgroups cut the array into contiguous
// ranges, the waves of a workgroup cut its range into contiguous ranges (the count and the split must agree on this).
__device__ __forceinline__ void wave_range(int64_t n, int blocks, int block, int wave, int64_t& first, int64_t& last) {
    const int64_t total = (n + kWaveChunk - 1) / kWaveChunk;
    const int64_t per_block = (total + blocks - 1) / blocks;
    const int64_t per_wave = (per_block + (kScanThreads / kWave) - 1) / (kScanThreads / kWave);
    const int64_t block_first = (int64_t)block * per_block;
    int64_t block_last = block_first + per_block;
    if (block_last > total) block_last = total;
    first = block_first + (int64_t)wave * per_wave;
    last = first + per_wave;
    if (first > block_last) first = block_last;
    if (last > block_last) last = block_last;
}

// The 8 requests of lane `lane` in the wave chunk starting at request `base`.
__device__ __forceinline__ void load_chunk(const SortDev& A, int64_t base, int lane, bool vec,
                                           uint32_t (&seg)[kScanItems], uint32_t (&key)[kScanItems],
                                           bool (&ok)[kScanItems]) {
    const PlanDev& P = A.plan;
#pragma unroll
    for (int g = 0; g < kScanItems / 4; ++g) {
        const int64_t r0 = lane_first(base, lane, g);
        int32_t d[4], st[4];
        if (vec && r0 + 3 < A.n) {
            const int4 d4 = *reinterpret_cast<const int4*>(A.deadline + r0);
            const int4 s4 = *reinterpret_cast<const int4*>(A.stage + r0);
            d[0] = d4.x; d[1] = d4.y; d[2] = d4.z; d[3] = d4.w;
            st[0] = s4.x; st[1] = s4.y; st[2] = s4.z; st[3] = s4.w;
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                d[c] = r0 + c < A.n ? A.deadline[r0 + c] : 0;
                st[c] = r0 + c < A.n ? A.stage[r0 + c] : 0;
            }
        }
        int32_t u = r0 < A.n ? snapshot_of(A.snap_ptr, P.K, r0) : 0;        // then forward: the four are consecutive
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int i = g * 4 + c;
            const int64_t r = r0 + c;
            ok[i] = r < A.n;
            while (ok[i] && u + 1 < P.K && r >= (int64_t)A.snap_ptr[u + 1]) ++u;
            const int32_t sidx = clamp_stage(st[c], P.S);
            const int32_t mode = P.uniform_mode >= 0 ? P.uniform_mode
                                                     : (P.recs[(P.shared ? 0 : (int64_t)u * P.S) + sidx].mode & 0xFF);
            const int32_t arr = (mode == PARD_ORDER_FCFS && ok[i]) ? A.arrival[r] : 0;
            seg[i] = (uint32_t)u * (uint32_t)P.S + (uint32_t)sidx;
            key[i] = order_key(mode, d[c], arr);
        }
    }
}

__device__ __forceinline__ bool arrays_vectorizable(const SortDev& A) {
    return ((reinterpret_cast<uintptr_t>(A.deadline) | reinterpret_cast<uintptr_t>(A.stage)) & 15) == 0;
}

// The same for a plan whose stages all order by deadline (MODE: low or high budget first) and that has at most
// 64 snapshots, without anything the general form needs only for other plans.  `bound` holds the snapshot
// boundaries across the lanes: lane k (1 <= k < K) has snap_ptr[k], every other lane INT32_MAX.
__device__ __forceinline__ int32_t snapshot_bound(const SortDev& A, int lane) {
    return lane >= 1 && lane < A.plan.K ? A.snap_ptr[lane] : kInt32Max;
}

template <int MODE>
__device__ __forceinline__ void load_chunk_by_deadline(const SortDev& A, int64_t base, int lane, bool vec, int32_t bound,
                                                       uint32_t (&snap)[kScanItems], uint32_t (&seg)[kScanItems],
                                                       uint32_t (&key)[kScanItems], bool (&ok)[kScanItems]) {
    const PlanDev& P = A.plan;
    int32_t d[kScanItems], st[kScanItems];
    if (vec && base + kWaveChunk <= A.n) {
#pragma unroll
        for (int g = 0; g < kScanItems / 4; ++g) {
            const int64_t r0 = lane_first(base, lane, g);
            const int4 d4 = *reinterpret_cast<const int4*>(A.deadline + r0);
            const int4 s4 = *reinterpret_cast<const int4*>(A.stage + r0);
            d[g * 4] = d4.x; d[g * 4 + 1] = d4.y; d[g * 4 + 2] = d4.z; d[g * 4 + 3] = d4.w;
            st[g * 4] = s4.x; st[g * 4 + 1] = s4.y; st[g * 4 + 2] = s4.z; st[g * 4 + 3] = s4.w;
        }
    } else {
#pragma unroll
        for (int i = 0; i < kScanItems; ++i) {
            const int64_t r = lane_first(base, lane, i / 4) + (i & 3);
            d[i] = r < A.n ? A.deadline[r] : 0;
            st[i] = r < A.n ? A.stage[r] : 0;
        }
    }
    // snapshot of the chunk's first request: the boundaries at or before it; then one step up per boundary inside
    const int32_t lo = (int32_t)base, hi = (int32_t)(base + kWaveChunk < A.n ? base + kWaveChunk : A.n);
    const uint32_t u_base = (uint32_t)__popcll(__ballot(bound <= lo));
    unsigned long long inside = __ballot(bound > lo && bound < hi);
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) snap[i] = u_base;
    while (inside) {
        const int32_t b = __builtin_amdgcn_readlane(bound, __builtin_ctzll(inside));
        inside &= inside - 1ull;
#pragma unroll
        for (int i = 0; i < kScanItems; ++i) snap[i] += (int32_t)(lane_first(base, lane, i / 4) + (i & 3)) >= b ? 1u : 0u;
    }
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) {
        ok[i] = lane_first(base, lane, i / 4) + (i & 3) < A.n;
        seg[i] = snap[i] * (uint32_t)P.S + (uint32_t)clamp_stage(st[i], P.S);
        key[i] = order_key(MODE, d[i], 0);
    }
}

// ---- count: queue lengths and key range ------------------------------------------
// No atomics on a shared global word here: every workgroup leaves its partial results in
// its own slot and the setup kernel adds them up.  (Same-address global atomics cost ~11 ns
// each on this chip and serialise.)
constexpr uint32_t kSawFall = 1u, kSawLongTie = 2u;
constexpr int kTieReach = 32;
constexpr int kCountLds = 16384;
constexpr int kCountPrivate = kCountLds / kScanThreads;    // up to 16 queues: one counter column per thread
// MODE: PARD_ORDER_LBF or PARD_ORDER_HBF when every stage orders that way and
// there are at most kPartialSegs queues (then the order of the deadlines is watched); -1 otherwise.
template <int MODE>
__global__ __launch_bounds__(kScanThreads, 8) void count_kernel(SortDev A) {
    __shared__ uint32_t h[kCountLds];
    __shared__ uint32_t red[2 * (kScanThreads / kWave)];
    __shared__ uint32_t saw_by_wave[kScanThreads / kWave];
    __shared__ uint32_t block_tot[kPartialSegs];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t segs = (int64_t)A.plan.K * A.plan.S;
    const bool priv = segs <= kCountPrivate;            // h[seg * 1024 + tid]: no two lanes share a counter
    const bool rows = !priv && segs <= kPartialSegs;    // h[wave * 64 + seg]: one row of counters per wave
    const bool use_lds = segs <= kCountLds;             // h[seg]: LDS atomics
    for (int i = tid; i < kCountLds; i += kScanThreads) h[i] = 0;
    if (tid < kPartialSegs) block_tot[tid] = 0;
    __syncthreads();
    const bool vec = arrays_vectorizable(A);
    uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
    // Does every snapshot come in deadline order (then its queues are a stable split by stage and nothing has to be
    // sorted)?  Only looked at when all stages order by deadline.  kSawFall: a deadline lower than the one before
    // it; kSawLongTie: more than kTieReach equal deadlines in a row (high budget first has to find the ends of a
    // run of equal deadlines, and looks no further than that).
    constexpr bool watch = MODE >= 0;
    const int32_t bound = watch ? snapshot_bound(A, lane) : 0;
    uint32_t saw = 0;
    int64_t first, last;
    wave_range(A.n, gridDim.x, blockIdx.x, wave, first, last);
    for (int64_t chunk = first; chunk < last; ++chunk) {
        const int64_t base = chunk * kWaveChunk;
        uint32_t seg[kScanItems], key[kScanItems];
        bool ok[kScanItems];
        if constexpr (!watch) load_chunk(A, base, lane, vec, seg, key, ok);
        if constexpr (watch) {
            uint32_t snap[kScanItems];
            // The deadline just before the chunk (lane 0) and, under high budget first, the ones kTieReach before
            // the lowest lanes' first requests are asked for here, so that they travel with the chunk's own loads
            // instead of costing a wait of their own each.
            int32_t d_before = 0, d_far = 0;
            const bool has_before = lane == 0 && base > 0 && base < A.n;
            if (has_before) d_before = A.deadline[base - 1];
            const int64_t r_far = lane_first(base, lane, 0) - kTieReach;
            const bool has_far = MODE == PARD_ORDER_HBF && lane < kTieReach / 4 && r_far >= 0 && r_far + kTieReach < A.n;
            if (has_far) d_far = A.deadline[r_far];
            load_chunk_by_deadline<MODE>(A, base, lane, vec, bound, snap, seg, key, ok);
            // the request before a lane's four: the last of the lane below; lane 0: the last request of the group
            // before, or for the chunk's first group the one in memory
#pragma unroll
            for (int g = 0; g < kScanItems / 4; ++g) {
                uint32_t before = __shfl_up(key[g * 4 + 3], 1), before_snap = __shfl_up(snap[g * 4 + 3], 1);
                if (g > 0) {
                    const uint32_t k63 = (uint32_t)__builtin_amdgcn_readlane((int)key[g * 4 - 1], 63);
                    const uint32_t s63 = (uint32_t)__builtin_amdgcn_readlane((int)snap[g * 4 - 1], 63);
                    if (lane == 0) { before = k63; before_snap = s63; }
                } else if (lane == 0) {
                    before = key[0];
                    before_snap = snap[0];
                    if (has_before) {
                        before = order_key(MODE, d_before, 0);
                        before_snap = (uint32_t)snapshot_of(A.snap_ptr, A.plan.K, base - 1);
                    }
                }
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int i = g * 4 + c;
                    if (!ok[i]) continue;
                    const uint32_t prev = c == 0 ? before : key[i - 1];
                    const uint32_t prev_snap = c == 0 ? before_snap : snap[i - 1];
                    // the key rises with the deadline under low budget first and falls with it under high budget first
                    if (snap[i] == prev_snap && (MODE == PARD_ORDER_LBF ? key[i] < prev : key[i] > prev)) saw |= kSawFall;
                }
            }
            if constexpr (MODE == PARD_ORDER_HBF) {
                // in sorted order, equal values kTieReach apart mean a run longer than that (a run of kTieReach + 4 or
                // more holds the first request of a group of four together with the one kTieReach before it); that
                // request is the first of the lane kTieReach / 4 below (lowest lanes: of the group before, or memory)
                static_assert(kTieReach % 4 == 0 && kTieReach / 4 < kWave, "the far request is a lane's first");
#pragma unroll
                for (int g = 0; g < kScanItems / 4; ++g) {
                    uint32_t far = __shfl_up(key[g * 4], kTieReach / 4);
                    if (g > 0) {
                        const uint32_t wrapped = (uint32_t)__shfl((int)key[g * 4 - 4], lane + kWave - kTieReach / 4);
                        if (lane < kTieReach / 4) far = wrapped;
                    } else if (lane < kTieReach / 4) {
                        far = ~key[g * 4];
                        if (has_far) far = order_key(MODE, d_far, 0);
                    }
                    if (ok[g * 4] && key[g * 4] == far) saw |= kSawLongTie;
                }
            }
        }
#pragma unroll
        for (int i = 0; i < kScanItems; ++i) {
            if (ok[i]) {
                if (priv) atomicAdd(&h[seg[i] * kScanThreads + tid], 1u);
                else if (rows) atomicAdd(&h[wave * kPartialSegs + seg[i]], 1u);
                else if (use_lds) atomicAdd(&h[seg[i]], 1u);
                else atomicAdd(&A.seg_count[seg[i]], 1u);
                kmin = key[i] < kmin ? key[i] : kmin;
                kmax = key[i] > kmax ? key[i] : kmax;
            }
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const uint32_t a = __shfl_xor(kmin, off), b = __shfl_xor(kmax, off);
        kmin = a < kmin ? a : kmin;
        kmax = b > kmax ? b : kmax;
    }
    if (lane == 0) { red[2 * wave] = ~kmin; red[2 * wave + 1] = kmax; }
    const uint32_t wave_saw = (__ballot(saw & kSawFall) ? kSawFall : 0u) | (__ballot(saw & kSawLongTie) ? kSawLongTie : 0u);
    if (lane == 0) saw_by_wave[wave] = wave_saw;
    // queue lengths of this wave's stretch, and of the workgroup's
    if (priv || rows) {
        uint32_t* mine = A.wave_cnt + ((int64_t)blockIdx.x * (kScanThreads / kWave) + wave) * kPartialSegs;
        if (priv) {
            for (int64_t g = 0; g < segs; ++g) {
                uint32_t v = h[g * kScanThreads + tid];
#pragma unroll
                for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
                if (lane == 0) { mine[g] = v; if (v) atomicAdd(&block_tot[g], v); }
            }
        } else {
            const uint32_t v = lane < segs ? h[wave * kPartialSegs + lane] : 0u;
            if (lane < segs) { mine[lane] = v; if (v) atomicAdd(&block_tot[lane], v); }
        }
    }
    __syncthreads();
    if (tid == 0) {
        uint32_t a = 0, b = 0, f = watch ? 0u : kSawFall;
        for (int w = 0; w < kScanThreads / kWave; ++w) {
            a = red[2 * w] > a ? red[2 * w] : a;
            b = red[2 * w + 1] > b ? red[2 * w + 1] : b;
            f |= saw_by_wave[w];
        }
        A.part_minmax[2 * blockIdx.x] = a;
        A.part_minmax[2 * blockIdx.x + 1] = b;
        A.part_flag[blockIdx.x] = f;
    }
    if (priv || rows) {
        if (tid < segs) A.part_cnt[(int64_t)blockIdx.x * kPartialSegs + tid] = block_tot[tid];
    } else if (use_lds) {
        for (int i = tid; i < segs; i += kScanThreads)
            if (h[i]) atomicAdd(&A.seg_count[i], h[i]);
    }
}

// ---- setup: one workgroup --------------------------------------------------------
__global__ __launch_bounds__(1024) void setup_kernel(SortDev A) {
    constexpr int kSlices = 1024 / kPartialSegs;
    __shared__ uint32_t wave_tot[16];
    __shared__ uint32_t carry;
    __shared__ uint32_t slice_tot[kSlices][kPartialSegs];
    const PlanDev& P = A.plan;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t segs = (int64_t)P.K * P.S;
    // Add up what the count kernel's workgroups left behind.  Everything that does not depend on anything else is
    // loaded first, in one go: key range and order flags per workgroup, and (up to kPartialSegs queues) the
    // workgroups' queue lengths, of which thread (slice, g) holds queue g of the workgroups [slice * len, (slice + 1) * len).
    __shared__ uint32_t mm[2][16];
    __shared__ uint32_t seen;
    __shared__ uint32_t qlen[kPartialSegs];
    __shared__ unsigned long long cfull_l[kPartialSegs];   // the stage costs at full queue length, when there are few queues
    constexpr int kHeld = 32;                             // per-workgroup counts a thread keeps in registers
    const bool few = segs <= kPartialSegs;
    const int g_mine = tid & (kPartialSegs - 1), slice = tid / kPartialSegs;
    const int len = (A.stream_blocks + kSlices - 1) / kSlices;
    const int b0 = slice * len, b1 = b0 + len < A.stream_blocks ? b0 + len : A.stream_blocks;
    uint32_t held[kHeld];
    uint32_t a = 0, b = 0, f = 0;
    for (int i = tid; i < A.stream_blocks; i += 1024) {
        const uint32_t x = A.part_minmax[2 * i], y = A.part_minmax[2 * i + 1];
        a = x > a ? x : a;
        b = y > b ? y : b;
        f |= A.part_flag[i];
    }
    uint32_t sum = 0;
    if (few) {
#pragma unroll
        for (int k = 0; k < kHeld; ++k) held[k] = b0 + k < b1 ? A.part_cnt[(int64_t)(b0 + k) * kPartialSegs + g_mine] : 0u;
#pragma unroll
        for (int k = 0; k < kHeld; ++k) sum += held[k];
        for (int bb = b0 + kHeld; bb < b1; ++bb) sum += A.part_cnt[(int64_t)bb * kPartialSegs + g_mine];
        slice_tot[slice][g_mine] = sum;
    }
    if (tid == 0) { seen = 0; carry = 0; }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const uint32_t x = __shfl_xor(a, off), y = __shfl_xor(b, off);
        a = x > a ? x : a;
        b = y > b ? y : b;
        f |= __shfl_xor(f, off);
    }
    if (lane == 0) { mm[0][wave] = a; mm[1][wave] = b; }
    __syncthreads();
    if (lane == 0 && f) atomicOr(&seen, f);
    if (few && tid < segs) {
        uint32_t v = 0;
        for (int sl = 0; sl < kSlices; ++sl) v += slice_tot[sl][tid];
        qlen[tid] = v;
        A.seg_count[tid] = v;
    }
    __syncthreads();
    // Requests in deadline order: the queues are a stable split by stage, done by split_kernel; the radix passes, the
    // epilogue and the unpacking then find nothing to do (passes = 0).
    const bool hbf = P.uniform_mode == PARD_ORDER_HBF;
    const bool in_order = A.n > 0 && few && !(seen & kSawFall) && !(hbf && (seen & kSawLongTie));
    const bool split = in_order && !A.consistent, presplit = in_order && A.consistent;
    if (tid == 0) {
        uint32_t inv_min = mm[0][0], max_key = mm[1][0];
        for (int w = 1; w < 16; ++w) {
            inv_min = mm[0][w] > inv_min ? mm[0][w] : inv_min;
            max_key = mm[1][w] > max_key ? mm[1][w] : max_key;
        }
        const uint32_t umin = ~inv_min;
        const uint32_t range = A.n > 0 ? max_key - umin : 0u;
        const uint32_t kb = 32u - (range ? (uint32_t)__clz((int)range) : 32u);
        const uint32_t total = kb + (uint32_t)A.seg_bits;
        const uint32_t passes = (total + kRadixBits - 1) / kRadixBits;
        A.params->inv_min = inv_min;
        A.params->max_key = max_key;
        A.params->kb = kb;
        A.params->total_bits = total;
        A.params->passes = (split || presplit) ? 0u : (passes < 1 ? 1u : passes);
        A.params->split = split ? 1u : 0u;
        A.params->presplit = presplit ? 1u : 0u;
    }
    if (split || presplit) {
        // a snapshot beyond the promised bound is flagged as the radix passes would flag it (their payload word
        // holds idx_bits of index); the split itself has no such limit
        for (int u = tid; u < P.K; u += 1024) {
            const int64_t size = (int64_t)A.snap_ptr[u + 1] - (int64_t)A.snap_ptr[u];
            if (A.idx_bits < 32 && size > ((int64_t)1 << A.idx_bits)) atomicOr(A.status_word, kStatusSnapshotTooLarge);
        }
        // part_cnt[b][g] becomes the number of requests of queue g in the workgroups before b
        uint32_t run = 0;
        for (int sl = 0; sl < slice; ++sl) run += slice_tot[sl][g_mine];
#pragma unroll
        for (int k = 0; k < kHeld; ++k) {
            if (b0 + k < b1) A.part_cnt[(int64_t)(b0 + k) * kPartialSegs + g_mine] = run;
            run += held[k];
        }
        for (int bb = b0 + kHeld; bb < b1; ++bb) {
            const uint32_t v = A.part_cnt[(int64_t)bb * kPartialSegs + g_mine];
            A.part_cnt[(int64_t)bb * kPartialSegs + g_mine] = run;
            run += v;
        }
    }
    __threadfence_block();           // nothing written so far is read by another workgroup of this kernel (there is none)
    __syncthreads();
    // queue offsets: exclusive scan of the queue lengths, 1024 at a time
    for (int64_t base = 0; base < segs + 1; base += 1024) {
        const int64_t g = base + tid;
        const uint32_t v = g < segs ? (few ? qlen[g] : __hip_atomic_load(&A.seg_count[g], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) : 0u;
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
        const uint64_t full = stage_cost(P.recs[rec], few ? qlen[g] : __hip_atomic_load(&A.seg_count[g], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT),
                                         P.lat + rec * PARD_LAT_ENTRIES);
        A.cfull[g] = full;
        if (few) cfull_l[g] = full;
    }
    // smallest execution latency of every queue: lat[min(B, a + 1)] over all positions a
    // (consistent dropping only)
    for (int64_t g = tid; g < segs && A.consistent; g += 1024) {
        const int64_t rec = P.shared ? g % P.S : g;
        const int32_t* row = P.lat + rec * PARD_LAT_ENTRIES;
        const int32_t B = P.recs[rec].B;
        uint32_t m = (uint32_t)row[0];
        bool rising = true;                              // then the cost never falls as the position grows
        for (int32_t b = 1; b < B; ++b) {
            m = (uint32_t)row[b] < m ? (uint32_t)row[b] : m;
            rising = rising && row[b] >= row[b - 1];
        }
        const bool by_deadline = (P.recs[rec].mode & 0xFF) != PARD_ORDER_FCFS;
        A.min_lat[g] = m | ((rising && by_deadline) ? kSegScan : 0u);
    }
    __threadfence_block();
    __syncthreads();
    // downstream maximum per (snapshot, stage): as given, or suffix sums along every path
    if (A.sub) {
        for (int64_t g = tid; g < segs; g += 1024) {
            const int64_t v = A.sub[g];
            A.down[g] = v < 0 ? 0ull : ((uint64_t)v < kCostCap ? (unsigned long long)v : (unsigned long long)kCostCap);
        }
        return;
    }
    const int64_t per_dag = P.dag_entry_ptr[1];                              // entries of the one shared DAG
    const int64_t items = P.shared ? per_dag * P.K : P.total_entries;        // (snapshot, path entry) pairs
    // Four pairs per thread at a time, each step of the walk issued for all four before any is used: with thousands of
    // queues this one workgroup has tens of thousands of pairs to walk, and a pair is a chain of dependent loads
    // (its snapshot, the end of its path, the stages behind it, their costs).
    constexpr int kPairs = 4;
    if (items <= 1024) {                     // a pair per thread at most: the plain walk
        const int64_t b = tid;
        if (b < items) {
            int32_t u, e;
            if (P.shared) { u = (int32_t)(b / per_dag); e = (int32_t)(b - (int64_t)u * per_dag); }
            else { e = (int32_t)b; u = P.entry_dag[e]; }
            const int32_t end = P.entry_end[e];
            unsigned long long sum = 0;
            for (int32_t t0 = e + 1; t0 < end; t0 += 8) {
                int32_t later[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) later[k] = t0 + k < end ? P.entry_stage[t0 + k] : -1;
#pragma unroll
                for (int k = 0; k < 8; ++k)
                    if (later[k] >= 0) sum += few ? cfull_l[(int64_t)u * P.S + later[k]] : A.cfull[(int64_t)u * P.S + later[k]];
            }
            atomicMax(&A.down[(int64_t)u * P.S + P.entry_stage[e]], sum);
        }
        return;
    }
    for (int64_t b0 = tid; b0 < items; b0 += 1024 * kPairs) {
        int32_t u[kPairs], e[kPairs], end[kPairs], own[kPairs];
        bool live[kPairs];
#pragma unroll
        for (int q = 0; q < kPairs; ++q) {
            const int64_t b = b0 + (int64_t)q * 1024;
            live[q] = b < items;
            u[q] = 0;
            e[q] = 0;
            if (live[q]) {
                if (P.shared) { u[q] = (int32_t)(b / per_dag); e[q] = (int32_t)(b - (int64_t)u[q] * per_dag); }
                else { e[q] = (int32_t)b; u[q] = P.entry_dag[e[q]]; }
            }
        }
#pragma unroll
        for (int q = 0; q < kPairs; ++q) {
            end[q] = live[q] ? P.entry_end[e[q]] : e[q] + 1;
            own[q] = live[q] ? P.entry_stage[e[q]] : 0;
        }
        unsigned long long sum[kPairs] = {0, 0, 0, 0};
        int32_t later[kPairs][8];
#pragma unroll
        for (int q = 0; q < kPairs; ++q)
#pragma unroll
            for (int k = 0; k < 8; ++k) later[q][k] = e[q] + 1 + k < end[q] ? P.entry_stage[e[q] + 1 + k] : -1;
#pragma unroll
        for (int q = 0; q < kPairs; ++q)
#pragma unroll
            for (int k = 0; k < 8; ++k)
                if (later[q][k] >= 0) sum[q] += few ? cfull_l[(int64_t)u[q] * P.S + later[q][k]] : A.cfull[(int64_t)u[q] * P.S + later[q][k]];
#pragma unroll
        for (int q = 0; q < kPairs; ++q) {
            // paths with more than eight stages behind the entry: the rest, eight ids in flight
            for (int32_t t0 = e[q] + 9; t0 < end[q]; t0 += 8) {
                int32_t more[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) more[k] = t0 + k < end[q] ? P.entry_stage[t0 + k] : -1;
#pragma unroll
                for (int k = 0; k < 8; ++k)
                    if (more[k] >= 0) sum[q] += few ? cfull_l[(int64_t)u[q] * P.S + more[k]] : A.cfull[(int64_t)u[q] * P.S + more[k]];
            }
            if (live[q]) atomicMax(&A.down[(int64_t)u[q] * P.S + own[q]], sum[q]);
        }
    }
}

// Digit `pass` of the virtual key  V = segment << kb | key  (key < 2^kb), without forming V: what the digit takes
// from the key and from the segment id are two shifts each, fixed for a whole pass.
struct DigitOf {
    uint32_t key_shift;             // the key contributes key >> key_shift (nothing when the digit starts at or above bit 32)
    uint32_t seg_left, seg_right;   // the segment contributes (segment << seg_left) >> seg_right
    uint32_t idx_bits;              // the segment id sits above this many bits of the payload word
    bool from_key, from_segment;
};

__device__ __forceinline__ DigitOf digit_plan(uint32_t kb, int pass, int idx_bits) {
    DigitOf D;
    const uint32_t sh = (uint32_t)(kRadixBits * pass);
    D.from_key = sh < 32u && sh < kb;
    D.key_shift = sh < 32u ? sh : 31u;
    D.from_segment = sh + kRadixBits > kb && idx_bits < 32;
    // a left shift of 8 or more leaves nothing of the segment inside the digit: 31 stands for all of them
    D.seg_left = kb > sh ? (kb - sh < 31u ? kb - sh : 31u) : 0u;
    D.seg_right = sh > kb ? (sh - kb < 31u ? sh - kb : 31u) : 0u;
    D.idx_bits = idx_bits < 32 ? (uint32_t)idx_bits : 31u;
    return D;
}

__device__ __forceinline__ uint32_t digit_of(const DigitOf& D, uint32_t key, uint32_t pay) {
    uint32_t v = D.from_key ? key >> D.key_shift : 0u;
    if (D.from_segment) v |= ((pay >> D.idx_bits) << D.seg_left) >> D.seg_right;
    return v & (kRadix - 1);
}

// exclusive scan of one value per thread over the radix-pass workgroup
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* tmp /*[kSortWaves]*/, int tid) {
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

// ---- one radix pass ----------------------------------------------------------------------
// Element e of a tile: wave w owns 1024 consecutive elements, item i lane l is element
// w*1024 + i*64 + l.
template <bool FIRST, int ITEMS>
__device__ __forceinline__ void load_tile(const SortDev& A, int pass, int64_t tile_base, int valid, int wave, int lane,
                                          uint32_t umin, bool need_pay, uint32_t (&key)[ITEMS], uint32_t (&pay)[ITEMS]) {
    constexpr int kSortItems = ITEMS;
    if (FIRST) {
        // every load is issued before the first key is formed (elements past the end re-read the
        // tile's first request and are zeroed afterwards)
        const PlanDev& P = A.plan;
        int32_t dl[kSortItems], st[kSortItems], ar[kSortItems];
#pragma unroll
        for (int i = 0; i < kSortItems; ++i) {
            const int e = wave * (kWave * kSortItems) + i * kWave + lane;
            const int64_t r = tile_base + (e < valid ? e : 0);
            dl[i] = A.deadline[r];
            st[i] = A.stage[r];
            ar[i] = P.any_fcfs ? A.arrival[r] : 0;
        }
        // most tiles lie inside one snapshot: its number and first request are then the same for
        // every element
        const int32_t u_first = snapshot_of(A.snap_ptr, P.K, tile_base);
        const int32_t u_last = snapshot_of(A.snap_ptr, P.K, tile_base + valid - 1);
        const int32_t first_of_u = A.snap_ptr[u_first];
        const uint32_t idx_mask = A.idx_bits < 32 ? (1u << A.idx_bits) - 1u : 0xFFFFFFFFu;
        uint32_t surplus = 0;
#pragma unroll
        for (int i = 0; i < kSortItems; ++i) {
            const int e = wave * (kWave * kSortItems) + i * kWave + lane;
            const int64_t r = tile_base + e;
            const bool ok = e < valid;
            const int32_t u = (ok && u_first != u_last) ? snapshot_between(A.snap_ptr, u_first, u_last, r) : u_first;
            const int32_t s = clamp_stage(st[i], P.S);
            const int32_t mode = P.uniform_mode >= 0 ? P.uniform_mode
                                                     : (P.recs[(P.shared ? 0 : (int64_t)u * P.S) + s].mode & 0xFF);
            const uint32_t seg = (uint32_t)u * (uint32_t)P.S + (uint32_t)s;
            const uint32_t k = order_key(mode, dl[i], mode == PARD_ORDER_FCFS ? ar[i] : 0);
            // index inside the snapshot; a snapshot larger than promised is flagged and its
            // surplus indices wrap (outputs unspecified then, never out of bounds)
            uint32_t local = ok ? (uint32_t)(r - (int64_t)(u_first != u_last ? A.snap_ptr[u] : first_of_u)) : 0u;
            surplus |= local & ~idx_mask;
            local &= idx_mask;
            key[i] = ok ? k - umin : 0u;
            pay[i] = ok ? (local | (A.idx_bits < 32 ? seg << A.idx_bits : 0u)) : 0u;
        }
        if (surplus) atomicOr(A.status_word, kStatusSnapshotTooLarge);
    } else {
        const uint32_t* src_key = A.key[(pass + 1) & 1];
        const uint32_t* src_pay = A.pay[(pass + 1) & 1];
#pragma unroll
        for (int i = 0; i < kSortItems; ++i) {
            const int e = wave * (kWave * kSortItems) + i * kWave + lane;
            key[i] = 0;
            pay[i] = 0;
            if (e < valid) {
                if (need_pay) {                 // the downsweep is the last reader of this buffer: streaming loads
                    key[i] = __builtin_nontemporal_load(src_key + tile_base + e);
                    pay[i] = __builtin_nontemporal_load(src_pay + tile_base + e);
                } else {
                    key[i] = src_key[tile_base + e];
                }
            }
        }
    }
}

// Upsweep: digit histogram of every tile, and of every chunk of kChunkTiles tiles.
template <bool FIRST, int ITEMS>
__global__ __launch_bounds__(kSortThreads, 4) void upsweep_kernel(SortDev A, int pass) {
    constexpr int kSortItems = ITEMS, kTile = kSortThreads * ITEMS;
    if (pass >= (int)A.params->passes) return;
    __shared__ uint32_t h[kRadix];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t umin = ~A.params->inv_min, kb = A.params->kb;
    const DigitOf dig = digit_plan(kb, pass, A.idx_bits);
    const bool need_pay = kRadixBits * (pass + 1) > (int)kb;      // the digit holds segment bits
    if (tid < kRadix) h[tid] = 0;
    __syncthreads();
    const int64_t tile = blockIdx.x;
    const int64_t tile_base = tile * kTile;
    const int valid = (int)((A.n - tile_base) < kTile ? (A.n - tile_base) : kTile);
    uint32_t key[kSortItems], pay[kSortItems];
    // A histogram does not care which element a lane holds: later passes read four consecutive
    // elements per lane with 16-byte loads (element (i/4)*256 + lane*4 + i%4 of the wave's 1024).
    const bool quads = !FIRST && valid == kTile;
    bool key_only = false;
    if (quads) {
        const uint32_t* src_key = A.key[(pass + 1) & 1];
        const uint32_t* src_pay = A.pay[(pass + 1) & 1];
#pragma unroll
        for (int g = 0; g < kSortItems / 4; ++g) {
            const int64_t at = tile_base + wave * (kWave * kSortItems) + g * (kWave * 4) + lane * 4;
            const uint4 kv = *reinterpret_cast<const uint4*>(src_key + at);
            key[4 * g] = kv.x; key[4 * g + 1] = kv.y; key[4 * g + 2] = kv.z; key[4 * g + 3] = kv.w;
            uint4 pv = make_uint4(0, 0, 0, 0);
            if (need_pay) pv = *reinterpret_cast<const uint4*>(src_pay + at);
            pay[4 * g] = pv.x; pay[4 * g + 1] = pv.y; pay[4 * g + 2] = pv.z; pay[4 * g + 3] = pv.w;
        }
    } else if (FIRST && !need_pay && A.plan.uniform_mode >= 0) {
        // One order for every stage and a digit without queue bits: the digit comes from the deadline (or the
        // arrival) alone, so neither the stage nor the snapshot of a request is looked at (half the bytes).
        const int32_t mode = A.plan.uniform_mode;
        const int32_t* src = mode == PARD_ORDER_FCFS ? A.arrival : A.deadline;
        const bool vec = valid == kTile && (reinterpret_cast<uintptr_t>(src) & 15) == 0;
#pragma unroll
        for (int g = 0; g < kSortItems / 4; ++g) {
            const int e0 = wave * (kWave * kSortItems) + g * (kWave * 4) + lane * 4;
            int32_t v[4];
            if (vec) {
                const int4 q = *reinterpret_cast<const int4*>(src + tile_base + e0);
                v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c) v[c] = e0 + c < valid ? src[tile_base + e0 + c] : 0;
            }
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                key[4 * g + c] = order_key(mode, v[c], v[c]) - umin;
                pay[4 * g + c] = e0 + c < valid ? 0u : 0xFFFFFFFFu;       // marks the elements past the end
            }
        }
        key_only = true;
    } else {
        load_tile<FIRST, ITEMS>(A, pass, tile_base, valid, wave, lane, umin, need_pay, key, pay);
    }
    bool runs = true;                          // this wave still looks for runs of one digit (below)
#pragma unroll
    for (int i = 0; i < kSortItems; ++i) {
        int e = quads ? 0 : wave * (kWave * kSortItems) + i * kWave + lane;       // a full tile: every element counts
        if (key_only) { e = pay[i] ? valid : 0; pay[i] = 0; }
        const uint32_t d = digit_of(dig, key[i], pay[i]);
        // Sorted input puts long runs of one digit into a wave, and 64 lanes adding to one LDS
        // word serialise: the two most common leading digits are counted with a ballot, the
        // remaining lanes add for themselves.  A wave that finds its digits spread out (the leading
        // digit shared by fewer than eight lanes) stops looking for runs: there the ballots only cost.
        unsigned long long todo = __ballot(e < valid);
        if (runs) {
#pragma unroll
            for (int round = 0; round < 2; ++round) {
                if (todo == 0ull) break;
                const int leader = __ffsll((long long)todo) - 1;
                const uint32_t d0 = (uint32_t)__builtin_amdgcn_readlane((int)d, leader);
                const unsigned long long same = __ballot(d == d0) & todo;
                if (lane == leader) atomicAdd(&h[d0], (uint32_t)__popcll(same));
                if (round == 0 && __popcll(same) < 8 && __popcll(todo) >= 32) runs = false;
                todo &= ~same;
            }
        }
        if ((todo >> lane) & 1ull) atomicAdd(&h[d], 1u);
    }
    __syncthreads();
    if (tid < kRadix) {
        const uint32_t c = h[tid];
        A.tile_hist[((int64_t)pass * A.tiles + tile) * kRadix + tid] = c;
        if (c) atomicAdd(&A.chunk_tot[((int64_t)pass * A.chunks + tile / kChunkTiles) * kRadix + tid], c);
    }
}

// One workgroup: chunk_tot[pass][c][d] (counts) -> first output slot of digit d in chunk c
// (scan over chunks inside a digit, digits in ascending order).
__global__ __launch_bounds__(1024) void digit_scan_kernel(SortDev A, int pass) {
    if (pass >= (int)A.params->passes) return;
    __shared__ uint32_t part[4][kRadix];
    __shared__ uint32_t base[kRadix];
    __shared__ uint32_t scan_tmp[16];
    const int tid = threadIdx.x, d = tid & (kRadix - 1), q = tid >> 8;           // quarter q of the chunks
    uint32_t* tot = A.chunk_tot + (int64_t)pass * A.chunks * kRadix;
    const int64_t per = (A.chunks + 3) / 4;
    const int64_t c_lo = q * per < A.chunks ? q * per : A.chunks, c_hi = c_lo + per < A.chunks ? c_lo + per : A.chunks;
    uint32_t sum = 0;
    for (int64_t c0 = c_lo; c0 < c_hi; c0 += 16) {      // 16 loads in flight
        uint32_t x[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) x[i] = c0 + i < c_hi ? tot[(c0 + i) * kRadix + d] : 0u;
#pragma unroll
        for (int i = 0; i < 16; ++i) sum += x[i];
    }
    part[q][d] = sum;
    __syncthreads();
    // exclusive scan over the 256 digit totals (threads 0..255 hold them; the others add zero)
    const int lane = tid & 63, wave = tid >> 6;
    const uint32_t v = q == 0 ? part[0][d] + part[1][d] + part[2][d] + part[3][d] : 0u;
    uint32_t inc = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t t = __shfl_up(inc, off);
        if (lane >= off) inc += t;
    }
    if (lane == 63) scan_tmp[wave] = inc;
    __syncthreads();
    if (q == 0) {
        uint32_t pre = 0;
        for (int w = 0; w < wave; ++w) pre += scan_tmp[w];
        base[d] = pre + inc - v;         // first output slot of digit d
    }
    __syncthreads();
    uint32_t run = base[d];
    for (int qq = 0; qq < q; ++qq) run += part[qq][d];
    for (int64_t c0 = c_lo; c0 < c_hi; c0 += 16) {      // a count is read and replaced by the same thread only
        uint32_t x[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) x[i] = c0 + i < c_hi ? tot[(c0 + i) * kRadix + d] : 0u;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            if (c0 + i < c_hi) tot[(c0 + i) * kRadix + d] = run;
            run += x[i];
        }
    }
}

// One workgroup per chunk: tile_hist[pass][t][d] (counts) -> first output slot of digit d of tile t.
// SCANNED: chunk_tot already holds every chunk's first slots (digit_scan_kernel ran).  Otherwise it
// holds counts and every workgroup derives its own first slots from all of them (few chunks).
template <bool SCANNED>
__global__ __launch_bounds__(kRadix) void chunk_scan_kernel(SortDev A, int pass) {
    if (pass >= (int)A.params->passes) return;
    __shared__ uint32_t scan_tmp[kRadix / kWave];
    const int d = threadIdx.x, lane = d & 63, wave = d >> 6;
    const int64_t c = blockIdx.x;
    const uint32_t* tot = A.chunk_tot + (int64_t)pass * A.chunks * kRadix;
    // the chunk's own tile counts do not depend on the chunk totals: all of these loads are issued before either is used
    const int64_t t_lo = c * kChunkTiles, t_hi = t_lo + kChunkTiles < A.tiles ? t_lo + kChunkTiles : A.tiles;
    uint32_t* th = A.tile_hist + (int64_t)pass * A.tiles * kRadix;
    uint32_t x[kChunkTiles];
#pragma unroll
    for (int i = 0; i < kChunkTiles; ++i) x[i] = t_lo + i < t_hi ? th[(t_lo + i) * kRadix + d] : 0u;
    uint32_t run;
    if (SCANNED) {
        run = tot[c * kRadix + d];
    } else {
        static_assert(kFusedScanChunks % 32 == 0, "the chunk totals of a digit are loaded in batches of 32");
        uint32_t all = 0, before = 0;
#pragma unroll
        for (int64_t c0 = 0; c0 < kFusedScanChunks; c0 += 32) {
            uint32_t y[32];
#pragma unroll
            for (int i = 0; i < 32; ++i) y[i] = c0 + i < A.chunks ? tot[(c0 + i) * kRadix + d] : 0u;
#pragma unroll
            for (int i = 0; i < 32; ++i) {
                all += y[i];
                if (c0 + i < c) before += y[i];
            }
        }
        uint32_t inc = all;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t t = __shfl_up(inc, off);
            if (lane >= off) inc += t;
        }
        if (lane == 63) scan_tmp[wave] = inc;
        __syncthreads();
        uint32_t pre = 0;
        for (int w = 0; w < wave; ++w) pre += scan_tmp[w];
        run = pre + inc - all + before;
    }
#pragma unroll
    for (int i = 0; i < kChunkTiles; ++i) {
        if (t_lo + i < t_hi) th[(t_lo + i) * kRadix + d] = run;
        run += x[i];
    }
}

// ---- epilogue: positions -> estimates, drop decisions, queue order ------------------------
// A request's queue position is its sorted position minus the start of its queue; with it come its own stage's
// cost, the downstream maximum and the decision.  The results are formed in queue order and belong in request
// order.  Written straight to their places, 4 bytes at a time and far from one another, every write reaches
// memory as a partial cache line (shuffled input: 37 bytes written per 4 bytes of payload).  So they go back in
// two steps.  The last radix pass does not write its keys out: it knows every element's final slot, forms the
// result there and then, writes the queue order (runs per digit, like the keys it would have written), and hands
// the pairs (request id, estimate | drop << 31) on gathered by the range of request ids they belong to: staged in
// LDS a second time and written as one run per range.  The order inside a range does not matter, so a tile
// reserves its place in every range with one atomic add (every id occurs once: a range holds exactly its share).
// A second kernel gives every range to one workgroup that puts each packed word at its request's place in LDS
// and writes the estimates and decisions of the range out in request order.  Up to kRetBuckets ranges of at most
// 2^kRetMaxShift ids; beyond that (more than 2^25 requests) the last pass writes its keys like any other, and
// epilogue_kernel scatters est | drop as ONE 4-byte write per request into the key buffer the last pass no
// longer needs, which unpack_kernel then streams out.
//
// With at most kEpiSegs queues everything a request needs about its queue (stage constants, queue start,
// downstream maximum, snapshot time) sits in LDS.
constexpr int kEpiSegs = 64;
constexpr int kEpiThreads = 256;

struct EpiSeg {                     // 80 bytes
    uint32_t B, W, latB, mode;
    uint32_t mB, shB, mW, shW;
    int32_t start, now;
    uint32_t down_lo, down_hi;
    int32_t first;                  // first request of the queue's snapshot
    int32_t len;                    // queue length
    uint32_t aux;                   // smallest execution latency | kSegScan << 31
    int32_t rec;                    // the queue's stage record and latency row in the plan
    uint32_t aW, bW;                // latB = aW * W + bW
    uint32_t pad[2];
};

// own-stage cost at queue position pos plus the downstream maximum: stage_cost() with the record
// held in registers
__device__ __forceinline__ uint64_t epilogue_estimate(const EpiSeg& q, const int32_t* lat_row, uint32_t pos) {
    const uint32_t batches = magic_div_dev(pos + q.B - 1u, q.mB, q.shB);
    const uint64_t p = (uint64_t)batches * q.bW;
    uint64_t wait = (uint64_t)batches * q.aW;
    if ((p >> 32) == 0) wait += magic_div_dev((uint32_t)p, q.mW, q.shW);
    else wait += wide_div(p, q.W);
    uint32_t ex = q.latB;
    if (pos + 1u < q.B) ex = (uint32_t)lat_row[pos];             // only the first B-1 requests of a queue
    uint64_t c = wait + ex;
    c = c < kCostCap ? c : kCostCap;
    return c + (((uint64_t)q.down_hi << 32) | q.down_lo);
}

// the deadline of request r back from its sort key (or from the input when the key is the arrival)
__device__ __forceinline__ int32_t epilogue_deadline(const SortDev& A, const EpiSeg& q, uint32_t key, uint32_t r, uint32_t umin) {
    const uint32_t uk = key + umin;
    const int32_t mode = (int32_t)(q.mode & 0xFF);
    if (mode == PARD_ORDER_LBF) return (int32_t)(uk ^ 0x80000000u);
    if (mode == PARD_ORDER_HBF) return (int32_t)(~uk ^ 0x80000000u);
    return (int64_t)r < A.n ? A.deadline[r] : 0;
}

__device__ __forceinline__ uint32_t epilogue_one(const SortDev& A, const EpiSeg& q, const int32_t* lat_row, int64_t j,
                                                 uint32_t key, uint32_t r, uint32_t umin) {
    const uint64_t e64 = epilogue_estimate(q, lat_row, (uint32_t)(j - (int64_t)q.start));
    int32_t est;
    uint8_t drp;
    finish_request(e64, q.now, epilogue_deadline(A, q, key, r, umin), est, drp);
    return (uint32_t)est | ((uint32_t)drp << 31);
}

__device__ __forceinline__ EpiSeg epilogue_segment(const SortDev& A, uint32_t seg) {
    const PlanDev& P = A.plan;
    const uint32_t u = seg / (uint32_t)P.S, k = seg - u * (uint32_t)P.S;
    const StageRec sr = P.recs[P.shared ? (int64_t)k : (int64_t)seg];
    const unsigned long long dn = A.down[seg];
    EpiSeg q;
    q.B = (uint32_t)sr.B; q.W = (uint32_t)sr.W; q.latB = (uint32_t)sr.latB; q.mode = (uint32_t)sr.mode;
    q.mB = sr.mB; q.shB = sr.shB; q.mW = sr.mW; q.shW = sr.shW;
    q.start = A.seg_ptr[seg]; q.now = A.now[u];
    q.first = A.snap_ptr[u];
    q.len = A.seg_ptr[seg + 1] - q.start;
    q.aux = A.consistent ? A.min_lat[seg] : 0u;
    q.rec = (int32_t)(P.shared ? k : seg);
    q.aW = sr.aW; q.bW = sr.bW; q.pad[0] = q.pad[1] = 0;
    q.down_lo = (uint32_t)dn; q.down_hi = (uint32_t)(dn >> 32);
    return q;
}

// request id and packed result (estimate | drop << 31) of queue slot j
__device__ __forceinline__ void epilogue_slot(const SortDev& A, const EpiSeg* tab, bool cached, int64_t j, uint32_t key,
                                              uint32_t pay, uint32_t umin, uint32_t idx_mask, uint32_t& r, uint32_t& out) {
    const PlanDev& P = A.plan;
    const uint32_t local = pay & idx_mask;
    const uint32_t seg = A.idx_bits < 32 ? (pay >> A.idx_bits) : 0u;
    if (cached) {
        const EpiSeg& q = tab[seg];
        r = (uint32_t)q.first + local;
        out = epilogue_one(A, q, P.lat + (int64_t)q.rec * PARD_LAT_ENTRIES, j, key, r, umin);
    } else {
        const EpiSeg q = epilogue_segment(A, seg);
        r = (uint32_t)q.first + local;
        out = epilogue_one(A, q, P.lat + (int64_t)q.rec * PARD_LAT_ENTRIES, j, key, r, umin);
    }
}

// Downsweep: rank the tile's elements among equal digits, reorder in LDS, write runs out.
template <bool FIRST, int ITEMS>
__global__ __launch_bounds__(kSortThreads, 4) void downsweep_kernel(SortDev A, int pass) {
    constexpr int kSortItems = ITEMS, kTile = kSortThreads * ITEMS;
    if (pass >= (int)A.params->passes) return;

    __shared__ uint32_t lds_key[kTile];
    __shared__ uint32_t lds_pay[kTile];
    __shared__ uint32_t whist[kSortWaves][kRadix];
    __shared__ uint32_t tile_start[kRadix];
    __shared__ uint32_t gbase[kRadix];
    __shared__ uint32_t scan_tmp[kSortWaves];
    __shared__ EpiSeg tab[kEpiSegs];                 // last pass only
    __shared__ uint32_t tile_total;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t umin = ~A.params->inv_min, kb = A.params->kb;
    const DigitOf dig = digit_plan(kb, pass, A.idx_bits);
    // the last pass forms the results instead of writing its keys out
    const bool finish = A.finish_in_last_pass && pass == (int)A.params->passes - 1;
    const bool cached = (int64_t)A.plan.K * A.plan.S <= kEpiSegs;
    if (finish && cached && tid < A.plan.K * A.plan.S) tab[tid] = epilogue_segment(A, (uint32_t)tid);
    uint32_t* dst_key = A.key[pass & 1];
    uint32_t* dst_pay = A.pay[pass & 1];
    for (int i = tid; i < kSortWaves * kRadix; i += kSortThreads) (&whist[0][0])[i] = 0;
    // Workgroups are handed to the 8 accelerator dies in turn.  Neighbouring tiles write
    // neighbouring runs of every digit, so each die takes a contiguous range of tiles: the
    // two halves of a cache line shared by two tiles then meet in the same L2.
    const int64_t per_die = (A.tiles + kDies - 1) / kDies;
    const int64_t tile = (int64_t)(blockIdx.x % kDies) * per_die + blockIdx.x / kDies;
    if (tile >= A.tiles) return;
    const int64_t tile_base = tile * kTile;
    const int valid = (int)((A.n - tile_base) < kTile ? (A.n - tile_base) : kTile);
    // first output slot of every digit of this tile
    const uint32_t first_slot = tid < kRadix ? A.tile_hist[((int64_t)pass * A.tiles + tile) * kRadix + tid] : 0u;

    uint32_t key[kSortItems], pay[kSortItems], rd[kSortItems];   // rd = rank | digit << 16
    load_tile<FIRST, ITEMS>(A, pass, tile_base, valid, wave, lane, umin, true, key, pay);
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kSortItems; ++i) {
        const int e = wave * (kWave * kSortItems) + i * kWave + lane;
        const bool ok = e < valid;
        const uint32_t d = digit_of(dig, key[i], pay[i]);
        // peers: the lanes that hold the same digit, found bit by bit.  Written on 32-bit halves as
        // peers & ~(vote ^ all) with all = every bit set when the lane's digit has bit b: one three-input
        // bit operation per half and bit (the 64-bit select it replaces took nine vector instructions per bit,
        // and this loop is what the kernel's time goes into).
        const unsigned long long live = __ballot(ok);
        uint32_t peers_lo = (uint32_t)live, peers_hi = (uint32_t)(live >> 32);
        // (the bits of the last digit above the key's top bit are zero in every lane: they vote alike and change nothing)
#pragma unroll
        for (int b = 0; b < kRadixBits; ++b) {
            const int32_t all = (int32_t)(d << (31 - b)) >> 31;
            const unsigned long long vote = __ballot(all < 0);
            // x & ~(y ^ z): truth table 0x90 of the three-input bit operation
            peers_lo = __builtin_amdgcn_bitop3_b32(peers_lo, (uint32_t)vote, (uint32_t)all, 0x90);
            peers_hi = __builtin_amdgcn_bitop3_b32(peers_hi, (uint32_t)(vote >> 32), (uint32_t)all, 0x90);
        }
        const uint32_t before = __builtin_amdgcn_mbcnt_hi(peers_hi, __builtin_amdgcn_mbcnt_lo(peers_lo, 0u));
        const uint32_t count = (uint32_t)(__popc(peers_lo) + __popc(peers_hi));
        uint32_t prev = 0;
        if (ok) {
            prev = whist[wave][d];
            if (before == count - 1) whist[wave][d] = prev + count;   // last peer advances the counter
        }
        rd[i] = (prev + before) | (d << 16);
    }
    __syncthreads();

    // per digit (threads 0..255): offsets of each wave's run inside the tile, tile count
    {
        const int d = tid & (kRadix - 1);
        const bool digit_thread = tid < kRadix;
        uint32_t run = 0;
        if (digit_thread) {
#pragma unroll
            for (int w = 0; w < kSortWaves; ++w) {
                const uint32_t t = whist[w][d];
                whist[w][d] = run;
                run += t;
            }
        }
        const uint32_t tstart = block_exclusive_scan(run, scan_tmp, tid);
        if (digit_thread) {
            tile_start[d] = tstart;
            gbase[d] = first_slot - tstart;
        }
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
    if (!finish) {
#pragma unroll
        for (int i = 0; i < kSortItems; ++i) {
            const int j = i * kSortThreads + tid;
            if (j < valid) {
                const uint32_t k = lds_key[j], p = lds_pay[j];
                const uint32_t d = digit_of(dig, k, p);
                const uint32_t dst = gbase[d] + (uint32_t)j;
                if ((int64_t)dst < A.n) { dst_key[dst] = k; dst_pay[dst] = p; }
            }
        }
        return;
    }

    // Last pass: element j of the reordered tile lands in queue slot gbase[digit] + j.
    uint32_t* first_place = &whist[0][0];            // results of the tile per range, then the range's first place in the tile
    uint32_t* delta = &whist[0][0] + kRetBuckets;    // the range's reserved place in memory minus its first place in the tile
    static_assert(2 * kRetBuckets <= kSortWaves * kRadix && kRetBuckets == 2 * kSortThreads, "the range counters reuse the digit counters, two ranges to a thread");
    const uint32_t idx_mask = A.idx_bits >= 32 ? 0xFFFFFFFFu : ((1u << A.idx_bits) - 1u);
    const int shift = A.ret_shift;
    const int64_t range = (int64_t)1 << shift;
    uint32_t r[kSortItems], out[kSortItems], rb[kSortItems];    // rb = place among the tile's results of its range | range << 16
    first_place[tid] = 0;                            // (the digit counters were last read before the barrier above)
    first_place[tid + kSortThreads] = 0;
#pragma unroll
    for (int i = 0; i < kSortItems; ++i) {
        const int j = i * kSortThreads + tid;
        r[i] = 0xFFFFFFFFu;
        out[i] = 0;
        if (j < valid) {
            const uint32_t k = lds_key[j], p = lds_pay[j];
            const uint32_t d = digit_of(dig, k, p);
            const uint32_t dst = gbase[d] + (uint32_t)j;
            if ((int64_t)dst < A.n) {
                epilogue_slot(A, tab, cached, (int64_t)dst, k, p, umin, idx_mask, r[i], out[i]);
                A.order[dst] = (int32_t)r[i];
            }
        }
    }
    __syncthreads();                                 // the tile's keys are out of LDS, the range counters are zero
    bool range_runs = true;
#pragma unroll
    for (int i = 0; i < kSortItems; ++i) {
        // a snapshot larger than promised can leave ids beyond the end: they are not returned
        const bool ok = (int64_t)r[i] < A.n;
        const uint32_t b = r[i] >> shift;
        // Input in arrival order puts one range into a whole wave, and 64 lanes adding to one LDS word serialise:
        // the most common range takes its places with one add.
        unsigned long long todo = __ballot(ok);
        uint32_t place = 0;
        if (todo != 0ull && range_runs) {
            const int leader = __ffsll((long long)todo) - 1;
            const uint32_t b0 = (uint32_t)__builtin_amdgcn_readlane((int)b, leader);
            const unsigned long long same = __ballot(b == b0) & todo;
            uint32_t old = 0;
            if (lane == leader) old = atomicAdd(&first_place[b0], (uint32_t)__popcll(same));
            old = (uint32_t)__builtin_amdgcn_readlane((int)old, leader);
            if ((same >> lane) & 1ull)
                place = old + __builtin_amdgcn_mbcnt_hi((uint32_t)(same >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)same, 0u));
            if (__popcll(same) < 8 && __popcll(todo) >= 32) range_runs = false;      // spread out: stop looking for runs
            todo &= ~same;
        }
        if ((todo >> lane) & 1ull) place = atomicAdd(&first_place[b], 1u);
        rb[i] = ok ? (place | (b << 16)) : 0xFFFFFFFFu;
    }
    __syncthreads();
    // Thread t takes ranges t and t + 512 (the second only exists beyond 2^24 requests): a range's first place in the
    // tile, and room for the tile's results in the range.  Both counts ride one scan, 16 bits each (a tile holds at
    // most 4096 results); the upper ranges come behind all the lower ones.  A wave's atomic adds cover 64
    // neighbouring counters, whole cache lines: two half-filled requests per line and tile (neighbouring ranges to a
    // thread) took the last pass from 146 to 203 us, the adds of all tiles to one line being served one after the other.
    {
        const uint32_t cnt0 = first_place[tid], cnt1 = first_place[tid + kSortThreads];
        const uint32_t before = block_exclusive_scan(cnt0 | (cnt1 << 16), scan_tmp, tid);
        uint32_t base0 = 0, base1 = 0;
        if (cnt0) base0 = atomicAdd(&A.ret_cursor[tid], cnt0);
        if (cnt1) base1 = atomicAdd(&A.ret_cursor[tid + kSortThreads], cnt1);
        uint32_t totals = 0;                         // the scan leaves every wave's total behind: both fields of the whole tile
#pragma unroll
        for (int w = 0; w < kSortWaves; ++w) totals += scan_tmp[w];
        const uint32_t lower_total = totals & 0xFFFFu;
        if (tid == 0) tile_total = lower_total + (totals >> 16);
        const uint32_t start0 = before & 0xFFFFu, start1 = lower_total + (before >> 16);
        first_place[tid] = start0;
        first_place[tid + kSortThreads] = start1;
        delta[tid] = base0 - start0;
        delta[tid + kSortThreads] = base1 - start1;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kSortItems; ++i) {
        if (rb[i] != 0xFFFFFFFFu) {
            const uint32_t lp = first_place[rb[i] >> 16] + (rb[i] & 0xFFFFu);
            lds_key[lp] = out[i];
            lds_pay[lp] = r[i];
        }
    }
    __syncthreads();
    const uint32_t total = tile_total;
#pragma unroll
    for (int i = 0; i < kSortItems; ++i) {
        const uint32_t j = (uint32_t)(i * kSortThreads + tid);
        if (j < total) {
            const uint32_t rr = lds_pay[j];
            const uint32_t b = rr >> shift;
            const int64_t first = (int64_t)b << shift;
            const int64_t room = A.n - first < range ? A.n - first : range;
            const uint32_t at = delta[b] + j;             // place inside the range
            if ((int64_t)at < room) {
                dst_pay[first + at] = rr;
                dst_key[first + at] = lds_key[j];
            }
        }
    }
}

// Order of the work.  Walking the queue slots front to back writes the packed results of one queue at a
// time, and the requests of a queue are spread over the whole request range: every cache line of packed[]
// is then written a few bytes at a time, as many times as there are queues, long after one another.  When
// the requests arrive roughly in key order (arrival-ordered input), the f-th fraction of every queue holds
// the requests of the same stretch of the request range.  So a workgroup takes one small share of EVERY queue
// at a time (share phi of `shares`: groups [L*phi/shares, L*(phi+1)/shares) of a queue that owns L groups of
// four slots): what it writes then falls into one stretch of packed[] and meets in its L2.
__global__ __launch_bounds__(kEpiThreads) void epilogue_kernel(SortDev A) {
    __shared__ EpiSeg tab[kEpiSegs];
    __shared__ int32_t gfirst[kEpiSegs + 1];     // first group of four slots a queue owns (the group's first slot is the queue's)
    __shared__ int32_t cum[kEpiSegs + 1];        // this share: groups of the queues before q
    __shared__ int32_t from[kEpiSegs];           // this share: its first group of queue q
    if (A.params->split) return;                 // the split kernel has written everything
    const PlanDev& P = A.plan;
    const int tid = threadIdx.x;
    const int64_t segs = (int64_t)P.K * P.S;
    const bool cached = segs <= kEpiSegs;
    if (cached && tid < segs) tab[tid] = epilogue_segment(A, (uint32_t)tid);
    __syncthreads();
    const int last = ((int)A.params->passes - 1) & 1;
    const uint32_t* keys = A.key[last];
    const uint32_t* pays = A.pay[last];
    uint32_t* packed = A.key[last ^ 1];
    const uint32_t umin = ~A.params->inv_min;
    const uint32_t idx_mask = A.idx_bits >= 32 ? 0xFFFFFFFFu : ((1u << A.idx_bits) - 1u);
    const bool vec = (reinterpret_cast<uintptr_t>(A.order) & 15) == 0;     // the workspace buffers are 256-byte aligned
    const int64_t groups = (A.n + 3) / 4;
    auto one_group = [&](const int64_t g) {
        const int64_t j0 = g * 4;
        uint32_t k4[4], p4[4];
        if (j0 + 3 < A.n) {
            const uint4 kv = *reinterpret_cast<const uint4*>(keys + j0);
            const uint4 pv = *reinterpret_cast<const uint4*>(pays + j0);
            k4[0] = kv.x; k4[1] = kv.y; k4[2] = kv.z; k4[3] = kv.w;
            p4[0] = pv.x; p4[1] = pv.y; p4[2] = pv.z; p4[3] = pv.w;
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                k4[c] = j0 + c < A.n ? keys[j0 + c] : 0u;
                p4[c] = j0 + c < A.n ? pays[j0 + c] : 0u;
            }
        }
        uint32_t r4[4], out[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            out[c] = 0;
            r4[c] = 0;
            if (j0 + c < A.n) epilogue_slot(A, tab, cached, j0 + c, k4[c], p4[c], umin, idx_mask, r4[c], out[c]);
        }
        if (vec && j0 + 3 < A.n) {
            *reinterpret_cast<int4*>(A.order + j0) = make_int4((int32_t)r4[0], (int32_t)r4[1], (int32_t)r4[2], (int32_t)r4[3]);
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (j0 + c < A.n) A.order[j0 + c] = (int32_t)r4[c];
        }
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (j0 + c < A.n && (int64_t)r4[c] < A.n) packed[r4[c]] = out[c];
    };
    if (!cached || segs < 2) {
        const int64_t stride = (int64_t)gridDim.x * kEpiThreads;
        for (int64_t g = (int64_t)blockIdx.x * kEpiThreads + tid; g < groups; g += stride) one_group(g);
        return;
    }
    if (tid <= segs) gfirst[tid] = tid < segs ? (int32_t)(((int64_t)tab[tid].start + 3) / 4) : (int32_t)groups;
    __syncthreads();
    const int64_t shares = (groups + kEpiThreads - kEpiSegs - 1) / (kEpiThreads - kEpiSegs);     // at most kEpiThreads groups each
    const int nseg = (int)segs;
    for (int64_t phi = blockIdx.x; phi < shares; phi += gridDim.x) {
        if (tid < kWave) {
            int32_t c = 0, f0 = 0;
            if (tid < nseg) {
                const int64_t L = gfirst[tid + 1] - gfirst[tid];
                const int64_t a0 = L * phi / shares, a1 = L * (phi + 1) / shares;
                c = (int32_t)(a1 - a0);
                f0 = gfirst[tid] + (int32_t)a0;
            }
            int32_t inc = c;
#pragma unroll
            for (int off = 1; off < kWave; off <<= 1) {
                const int32_t t = __shfl_up(inc, off);
                if (tid >= off) inc += t;
            }
            if (tid < nseg) { cum[tid] = inc - c; from[tid] = f0; }
            if (tid == nseg - 1) cum[nseg] = inc;
        }
        __syncthreads();
        const int total = cum[nseg];
        for (int x = tid; x < total; x += kEpiThreads) {
            int lo = 0, hi = nseg;                       // the last queue with cum[q] <= x holds x
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (cum[mid] <= x) lo = mid; else hi = mid;
            }
            one_group((int64_t)from[lo] + (x - cum[lo]));
        }
        __syncthreads();
    }
}

__global__ __launch_bounds__(256) void unpack_kernel(SortDev A) {
    if (A.params->split) return;
    const uint32_t* packed = A.key[(((int)A.params->passes - 1) & 1) ^ 1];
    const bool vec = ((reinterpret_cast<uintptr_t>(A.est) & 15) | (reinterpret_cast<uintptr_t>(A.drop) & 3)) == 0;
    const int64_t groups = (A.n + 3) / 4;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < groups; g += stride) {
        const int64_t r0 = g * 4;
        if (vec && r0 + 3 < A.n) {
            // read once, written once: streaming accesses
            const pard_v4i v_ = __builtin_nontemporal_load(reinterpret_cast<const pard_v4i*>(packed + r0));
            const uint4 v = make_uint4((uint32_t)v_.x, (uint32_t)v_.y, (uint32_t)v_.z, (uint32_t)v_.w);
            stream_store(reinterpret_cast<int4*>(A.est + r0), make_int4((int32_t)(v.x & 0x7FFFFFFFu), (int32_t)(v.y & 0x7FFFFFFFu),
                                                             (int32_t)(v.z & 0x7FFFFFFFu), (int32_t)(v.w & 0x7FFFFFFFu)));
            *reinterpret_cast<uint32_t*>(A.drop + r0) = (v.x >> 31) | ((v.y >> 31) << 8) | ((v.z >> 31) << 16) | ((v.w >> 31) << 24);
        } else {
            for (int64_t r = r0; r < r0 + 4 && r < A.n; ++r) {
                const uint32_t v = packed[r];
                A.est[r] = (int32_t)(v & 0x7FFFFFFFu);
                A.drop[r] = (uint8_t)(v >> 31);
            }
        }
    }
}

// Second step of the way back to request order: one workgroup per range of request ids.
template <int SHIFT, int kRetWgThreads>
__global__ __launch_bounds__(kRetWgThreads) void epilogue_return_kernel(SortDev A) {
    constexpr int kRetShift = SHIFT, kRetRange = 1 << SHIFT;
    __shared__ uint32_t by_request[kRetRange];
    if (A.params->split) return;
    const int last = ((int)A.params->passes - 1) & 1;            // where the last pass would have written its keys
    const uint32_t* ret_out = A.key[last];
    const uint32_t* ret_r = A.pay[last];
    const int tid = threadIdx.x;
    const int64_t first = (int64_t)blockIdx.x << kRetShift;
    if (first >= A.n) return;
    const int room = (int)(A.n - first < kRetRange ? A.n - first : kRetRange);
    // A range holds exactly its share of results unless a snapshot broke its promise, so the loads do not wait for the
    // count: they cover the range's whole room (all of it inside the buffer), and the count only decides which of the
    // words loaded are results.
    int cnt = (int)A.ret_cursor[blockIdx.x];
    if (cnt > room) cnt = room;
    constexpr int kAhead = 4;                                   // groups of four per thread in flight
    for (int i0 = tid * 4; i0 < room; i0 += kRetWgThreads * 4 * kAhead) {
        uint32_t rr[kAhead][4], oo[kAhead][4];
#pragma unroll
        for (int a = 0; a < kAhead; ++a) {
            const int i = i0 + a * kRetWgThreads * 4;
            if (i + 3 < room) {
                const pard_v4i rv = __builtin_nontemporal_load(reinterpret_cast<const pard_v4i*>(ret_r + first + i));
                const pard_v4i ov = __builtin_nontemporal_load(reinterpret_cast<const pard_v4i*>(ret_out + first + i));
                rr[a][0] = (uint32_t)rv.x; rr[a][1] = (uint32_t)rv.y; rr[a][2] = (uint32_t)rv.z; rr[a][3] = (uint32_t)rv.w;
                oo[a][0] = (uint32_t)ov.x; oo[a][1] = (uint32_t)ov.y; oo[a][2] = (uint32_t)ov.z; oo[a][3] = (uint32_t)ov.w;
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    rr[a][c] = i + c < room ? ret_r[first + i + c] : 0u;
                    oo[a][c] = i + c < room ? ret_out[first + i + c] : 0u;
                }
            }
        }
#pragma unroll
        for (int a = 0; a < kAhead; ++a) {
            const int i = i0 + a * kRetWgThreads * 4;
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (i + c < cnt) by_request[rr[a][c] & (kRetRange - 1)] = oo[a][c];      // the id lies in this range
        }
    }
    __syncthreads();
    const bool vec = ((reinterpret_cast<uintptr_t>(A.est) & 15) | (reinterpret_cast<uintptr_t>(A.drop) & 3)) == 0;
    for (int i = tid * 4; i < room; i += kRetWgThreads * 4) {
        if (vec && i + 3 < room) {
            const uint4 v = *reinterpret_cast<const uint4*>(&by_request[i]);
            stream_store(reinterpret_cast<int4*>(A.est + first + i), make_int4((int32_t)(v.x & 0x7FFFFFFFu), (int32_t)(v.y & 0x7FFFFFFFu),
                                                                                  (int32_t)(v.z & 0x7FFFFFFFu), (int32_t)(v.w & 0x7FFFFFFFu)));
            *reinterpret_cast<uint32_t*>(A.drop + first + i) = (v.x >> 31) | ((v.y >> 31) << 8) | ((v.z >> 31) << 16) | ((v.w >> 31) << 24);
        } else {
            for (int c = 0; c < 4 && i + c < room; ++c) {
                const uint32_t v = by_request[i + c];
                A.est[first + i + c] = (int32_t)(v & 0x7FFFFFFFu);
                A.drop[first + i + c] = (uint8_t)(v >> 31);
            }
        }
    }
}

// ---- split: snapshots whose requests come in deadline order ----------------------------------
// When the deadlines never fall along the request array (a queue snapshot taken in arrival order, one SLO), the
// queue order needs no sort.  Low budget first: a queue holds its requests in request order, so a request's
// position is the number of earlier requests of its stage.  High budget first: the reverse, except that requests
// with equal deadlines keep their request order: with j earlier requests of the stage, `before` of them and
// `after` later ones sharing the deadline, the position is (queue length - 1 - j) - after + before.  Equal
// deadlines are neighbours in the array, so before and after come from looking left and right as long as the
// deadline stays the same (the count kernel has ruled out runs longer than kTieSearch).
// Every wave takes the same contiguous stretch of the array as in the count kernel and works on its own: lane g
// starts from the number of requests of queue g before the stretch (workgroups before: left by the setup kernel;
// waves before in the workgroup: the count kernel's per-wave counts) and carries it along.  Estimates and
// decisions leave in request order (coalesced); only the queue order is scattered, as one ascending or
// descending stream per queue.  Under high budget first a wave keeps the keys and queues of its 512 requests,
// and of kTieSearch requests on either side, in its own piece of LDS for the look to the left and right.
constexpr int kTieSearch = 40;
constexpr int kSplitWaves = kScanThreads / kWave;      // waves per workgroup of the count kernel
constexpr int kSplitThreads = 256;                     // the split's own workgroups: a quarter of those waves each
constexpr int kSplitPerCount = kScanThreads / kSplitThreads;
constexpr int kHaloSpan = kWaveChunk + 2 * kTieSearch;

// OR over the 64 lanes of a wave (the result is the same in every lane's copy of the return value)
__device__ __forceinline__ uint32_t wave_or(uint32_t v) {
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xF, 0xF, false);    // row_shr:1
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xF, 0xF, false);    // row_shr:2
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xF, 0xF, false);    // row_shr:4
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xF, 0xF, false);    // row_shr:8
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xA, 0xF, false);    // row_bcast:15 into rows 1, 3
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xC, 0xF, false);    // row_bcast:31 into rows 2, 3
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// Queues are counted three to a 32-bit word, ten bits each: a wave chunk holds 512 requests, so no field passes 512.
constexpr uint32_t kFieldBits = 10, kFieldMask = (1u << kFieldBits) - 1u;
constexpr uint32_t kNoWord = 31;

// CONS (sequentially consistent dropping): nothing is decided here; the sort key and payload of every request go
// to its queue slot in the buffers the consistent_* kernels read (those of an odd last pass: no pass has run).
template <bool HBF, bool CONS>
__global__ __launch_bounds__(kSplitThreads) void split_kernel(SortDev A) {
    if (!(CONS ? A.params->presplit : A.params->split)) return;
    __shared__ EpiSeg tab[kPartialSegs];
    __shared__ __align__(16) uint32_t halo_key[HBF ? kSplitThreads / kWave : 1][HBF ? kHaloSpan : 4];
    __shared__ __align__(16) uint8_t halo_seg[HBF ? kSplitThreads / kWave : 1][HBF ? kHaloSpan : 16];
    const PlanDev& P = A.plan;
    const int tid = threadIdx.x, lane = tid & 63, own = tid >> 6;
    // which workgroup and wave of the count kernel this wave follows
    const int block = blockIdx.x / kSplitPerCount, wave = (blockIdx.x % kSplitPerCount) * (kSplitThreads / kWave) + own;
    const int blocks = gridDim.x / kSplitPerCount;
    const int segs = P.K * P.S;
    if (tid < segs) tab[tid] = epilogue_segment(A, (uint32_t)tid);
    // lane g: requests of queue g before this wave's stretch
    uint32_t run = 0;
    if (lane < segs) {
        run = A.part_cnt[(int64_t)block * kPartialSegs + lane];
        const uint32_t* rows = A.wave_cnt + (int64_t)block * kSplitWaves * kPartialSegs + lane;
        uint32_t v[kSplitWaves - 1];
#pragma unroll
        for (int w = 0; w < kSplitWaves - 1; ++w) v[w] = w < wave ? rows[w * kPartialSegs] : 0u;
#pragma unroll
        for (int w = 0; w < kSplitWaves - 1; ++w) run += v[w];
    }
    const uint32_t lane_word = ((uint32_t)lane * 43u) >> 7;             // lane / 3 (exact below 128)
    const uint32_t lane_shift = kFieldBits * ((uint32_t)lane - 3u * lane_word);
    const bool vec = arrays_vectorizable(A);
    const bool vec_out = ((reinterpret_cast<uintptr_t>(A.est) & 15) | (reinterpret_cast<uintptr_t>(A.drop) & 3)) == 0;
    const int32_t bound = snapshot_bound(A, lane);
    const uint32_t umin = ~A.params->inv_min;
    const uint32_t idx_mask = A.idx_bits >= 32 ? 0xFFFFFFFFu : ((1u << A.idx_bits) - 1u);
    int64_t first, last;
    wave_range(A.n, blocks, block, wave, first, last);
    __syncthreads();
    for (int64_t chunk = first; chunk < last; ++chunk) {
        const int64_t base = chunk * kWaveChunk;
        uint32_t snap[kScanItems], seg[kScanItems], key[kScanItems], j[kScanItems];
        bool ok[kScanItems];
        // (the neighbours on either side of the chunk, needed under high budget first, are asked for before the chunk
        // itself so that all of them travel together: a wait of their own per chunk otherwise)
        int32_t halo_d[2] = {0, 0}, halo_st[2] = {0, 0};
        if constexpr (HBF) {
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int h = lane + t * kWave;
                const int64_t r = h < kTieSearch ? base - kTieSearch + h : base + kWaveChunk + (h - kTieSearch);
                if (h < 2 * kTieSearch && r >= 0 && r < A.n) { halo_d[t] = A.deadline[r]; halo_st[t] = A.stage[r]; }
            }
        }
        load_chunk_by_deadline<HBF ? PARD_ORDER_HBF : PARD_ORDER_LBF>(A, base, lane, vec, bound, snap, seg, key, ok);
        // same queue, same deadline, to the left / right of a request: among the lane's own four, and beyond them (a byte each)
        uint32_t near_before[kScanItems] = {0, 0, 0, 0, 0, 0, 0, 0}, near_after[kScanItems] = {0, 0, 0, 0, 0, 0, 0, 0};
        uint64_t ties_before = 0, ties_after = 0;
        if constexpr (HBF) {
            // the neighbours on either side of the wave chunk (two loads per lane at most), then the chunk itself
            uint32_t* hk = halo_key[own];
            uint8_t* hs = halo_seg[own];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int h = lane + t * kWave;                                   // 0 .. 127, of which 2 * kTieSearch used
                if (h < 2 * kTieSearch) {
                    const bool left = h < kTieSearch;
                    const int64_t r = left ? base - kTieSearch + h : base + kWaveChunk + (h - kTieSearch);
                    const int at = left ? h : kTieSearch + kWaveChunk + (h - kTieSearch);
                    uint32_t k = 0, sg = 0xFFu;
                    if (r >= 0 && r < A.n) {
                        k = order_key(PARD_ORDER_HBF, halo_d[t], 0);
                        const uint32_t u = P.K == 1 ? 0u : (uint32_t)snapshot_of(A.snap_ptr, P.K, r);
                        sg = u * (uint32_t)P.S + (uint32_t)clamp_stage(halo_st[t], P.S);
                    }
                    hk[at] = k;
                    hs[at] = (uint8_t)sg;
                }
            }
            // a lane's four keys of group g sit at kTieSearch + 256 g + 4 lane (a 16-byte boundary)
            static_assert(kTieSearch % 4 == 0, "a lane's four keys sit on a 16-byte boundary");
            const int at0 = kTieSearch + lane * 4;
#pragma unroll
            for (int g = 0; g < kScanItems / 4; ++g) {
                *reinterpret_cast<uint4*>(hk + at0 + g * kGroupSpan) = make_uint4(key[g * 4], key[g * 4 + 1], key[g * 4 + 2], key[g * 4 + 3]);
                uint32_t four = 0;
#pragma unroll
                for (int c = 0; c < 4; ++c) four |= (ok[g * 4 + c] ? seg[g * 4 + c] : 0xFFu) << (8 * c);
                *reinterpret_cast<uint32_t*>(hs + at0 + g * kGroupSpan) = four;
            }
            // the wave's own LDS traffic runs in order; this only keeps the compiler from moving reads above the writes
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            // Same queue and same deadline among the lane's own four: every pair counts once to the left and once
            // to the right (the deadlines are sorted, so equal ends mean an equal stretch).  Only a run that reaches
            // past the lane's four needs a look into LDS, from the lane's edge outwards.
            uint32_t looks = 0;                                  // bit i: look left for request i, bit 8 + i: right
#pragma unroll
            for (int g = 0; g < kScanItems / 4; ++g) {
                const bool edge_left = hk[at0 + g * kGroupSpan - 1] == key[g * 4];
                const bool edge_right = hk[at0 + g * kGroupSpan + 4] == key[g * 4 + 3];
#pragma unroll
                for (int a = 0; a < 4; ++a)
#pragma unroll
                    for (int b = a + 1; b < 4; ++b) {
                        const uint32_t both = (ok[g * 4 + b] && key[g * 4 + a] == key[g * 4 + b] && seg[g * 4 + a] == seg[g * 4 + b]) ? 1u : 0u;
                        near_before[g * 4 + b] += both;
                        near_after[g * 4 + a] += both;
                    }
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    looks |= ((edge_left && key[g * 4] == key[g * 4 + c]) ? 1u : 0u) << (g * 4 + c);
                    looks |= ((edge_right && key[g * 4 + 3] == key[g * 4 + c]) ? 1u : 0u) << (kScanItems + g * 4 + c);
                }
            }
            // one look at a time (rare: deadlines are in microseconds), a byte of the result per request
            while (looks) {
                const int b = __builtin_ctz(looks);
                looks &= looks - 1u;
                const int i = b & (kScanItems - 1), step = b < kScanItems ? -1 : 1;
                const int mine = at0 + (i >> 2) * kGroupSpan;
                const uint32_t uk = hk[mine + (i & 3)];
                const uint8_t sg = hs[mine + (i & 3)];
                const int from = step < 0 ? mine - 1 : mine + 4;    // the first request beyond the lane's four
                uint32_t same = 0;
                for (int t = 0; t < kTieSearch; ++t) {
                    if (hk[from + step * t] != uk) break;
                    same += hs[from + step * t] == sg ? 1u : 0u;
                }
                if (step < 0) ties_before |= (uint64_t)same << (8 * i);
                else ties_after |= (uint64_t)same << (8 * i);
            }
        }
        // j: requests of the same queue ahead in the array.  First those before the chunk ...
        uint32_t word[kScanItems], shift[kScanItems], present = 0;
#pragma unroll
        for (int i = 0; i < kScanItems; ++i) {
            j[i] = (uint32_t)__shfl((int)run, (int)(seg[i] & 63u));
            const uint32_t w = (seg[i] * 43u) >> 7;                      // seg / 3
            shift[i] = kFieldBits * (seg[i] - 3u * w);
            word[i] = ok[i] ? w : kNoWord;
            present |= 1u << word[i];
        }
        // ... then, word by word of three queues, those earlier in the chunk: the group before, lower lanes of the own
        // group, and earlier ones among the lane's own four
        uint32_t words = wave_or(present) & ~(1u << kNoWord);
        while (words) {
            const uint32_t w = (uint32_t)__builtin_ctz(words);
            words &= words - 1u;
            uint32_t earlier = 0;                                // the groups before, all lanes
#pragma unroll
            for (int g = 0; g < kScanItems / 4; ++g) {
                uint32_t partial[5];
                partial[0] = 0;
#pragma unroll
                for (int c = 0; c < 4; ++c) partial[c + 1] = partial[c] + (word[g * 4 + c] == w ? 1u << shift[g * 4 + c] : 0u);
                const uint32_t inclusive = wave_inclusive_sum(partial[4]);
                const uint32_t below = earlier + inclusive - partial[4];
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (word[g * 4 + c] == w) j[g * 4 + c] += ((below + partial[c]) >> shift[g * 4 + c]) & kFieldMask;
                earlier += (uint32_t)__builtin_amdgcn_readlane((int)(inclusive - partial[4]), 63) +
                           (uint32_t)__builtin_amdgcn_readlane((int)partial[4], 63);
            }
            if (lane_word == w) run += (earlier >> lane_shift) & kFieldMask;
        }
#pragma unroll
        for (int g = 0; g < kScanItems / 4; ++g) {
            const int64_t r0 = lane_first(base, lane, g);
            int32_t est[4];
            uint8_t drp[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int i = g * 4 + c;
                est[c] = 0;
                drp[c] = 0;
                if (!ok[i]) continue;
                const int64_t r = r0 + c;
                const EpiSeg& q = tab[seg[i]];
                const uint32_t uk = key[i];
                const int32_t d = HBF ? (int32_t)(~uk ^ 0x80000000u) : (int32_t)(uk ^ 0x80000000u);
                uint32_t pos = j[i];
                if constexpr (HBF) {
                    // requests of the same queue with the same deadline right before and right after this one
                    const uint32_t before = near_before[i] + ((uint32_t)(ties_before >> (8 * i)) & 0xFFu);
                    const uint32_t after = near_after[i] + ((uint32_t)(ties_after >> (8 * i)) & 0xFFu);
                    pos = (uint32_t)q.len - 1u - j[i] - after + before;
                }
                if constexpr (CONS) {
                    const int64_t slot = (int64_t)q.start + pos;
                    if (slot < A.n) {
                        A.key[1][slot] = uk - umin;
                        A.pay[1][slot] = ((uint32_t)(r - (int64_t)q.first) & idx_mask) | (A.idx_bits < 32 ? seg[i] << A.idx_bits : 0u);
                    }
                    continue;
                }
                const uint64_t e64 = epilogue_estimate(q, P.lat + (int64_t)q.rec * PARD_LAT_ENTRIES, pos);
                finish_request(e64, q.now, d, est[c], drp[c]);
                A.order[(int64_t)q.start + pos] = (int32_t)r;
            }
            if constexpr (CONS) continue;
            if (vec_out && r0 + 3 < A.n) {
                // (the decisions are stored normally: the streamed compaction gathers them right afterwards)
                stream_store(reinterpret_cast<int4*>(A.est + r0), make_int4(est[0], est[1], est[2], est[3]));
                *reinterpret_cast<uint32_t*>(A.drop + r0) =
                    (uint32_t)drp[0] | ((uint32_t)drp[1] << 8) | ((uint32_t)drp[2] << 16) | ((uint32_t)drp[3] << 24);
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (ok[g * 4 + c]) { A.est[r0 + c] = est[c]; A.drop[r0 + c] = drp[c]; }
            }
        }
        if constexpr (HBF) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
    }
}

// ---- sequentially consistent dropping on sorted queues --------------------------------------
// A request's position counts only the kept requests ahead of it (the Request Broker takes a
// queue in order and a dropped request never takes a batch slot, paper Section 4.1), so every
// queue is one chain of decisions:  a_0 = 0,  a_{i+1} = a_i + [request i is kept at position a_i].
//
// Queues ordered by deadline whose cost never falls with the position (latency table rising up
// to the batch size) need no chain.  Let c_i be the number of positions at which request i
// would still be in time (they form a prefix 0..c_i-1), so request i is kept iff a_i < c_i.
//   Low budget first:  budgets rise along the queue, so c_i never falls, a_i <= c_i always
//   holds and the recurrence is a_{i+1} = min(a_i + 1, c_i), i.e.
//        a_i = min(i, i - 1 + min over i' < i of (c_i' - i'))        an exclusive prefix minimum.
//   High budget first:  c_i never rises; the kept requests are exactly the leading ones that the
//   plain rule (position = i) keeps, so  a_i = min(i, first i' < i with i' >= c_i').
// Both are segmented exclusive prefix minima over the queue slots: per-tile totals from the
// prepare kernel (whose workgroups each own a range of tiles and carry the scan across it), one
// small scan over the ranges, and the finish kernel redoes the scan inside its tile.  c_i has a closed form (positions_in_time).
//
// Any other queue (arrival order, or a latency table that falls somewhere) is walked:
//   prepare   also leaves one bit per slot that says whether the request could be kept at all,
//             i.e. at the smallest cost any position can have; in an overloaded queue most
//             requests fail that test, and they are dropped whatever happens ahead of them
//   chain     one wave per such queue walks the words of that bit mask in order, skipping
//             words without candidates; the 64 slots of a word are settled together by
//             iterating the decisions to their fixed point (after t rounds the first t lanes are
//             final); it leaves the keep bits and, per mask word, the kept requests before it
//   finish    position = kept requests ahead from the keep bits.
// In both cases prepare replaces the sort key by the deadline in place, and finish ends like the
// plain epilogue: estimate and drop decision at the position found.
constexpr int kChainWords = 64;                         // mask words (of 64 slots) a chain step looks at
constexpr int kChainAhead = 32;                         // steps whose mask words are in flight together
constexpr int32_t kNoMin = 0x7fffffff;

// Number of positions a in [0, queue length) at which a request with T microseconds left for
// its own stage (deadline - now - downstream) is in time, for a cost that never falls with a.
__device__ __forceinline__ uint32_t positions_in_time(const EpiSeg& q, const int32_t* lat_row, int64_t T) {
    const uint32_t L = (uint32_t)q.len;
    if (T < 0) return 0u;
    const uint32_t w1 = magic_div_dev(q.latB, q.mW, q.shW);      // floor(lat[B] / W): the wait behind one batch
    const uint32_t r1 = L < q.B - 1u ? L : q.B - 1u;              // positions that see a partial batch
    uint32_t lo = 0, hi = r1;                                     // first late position among them
    while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        const uint64_t c = (uint64_t)(mid ? w1 : 0u) + (uint32_t)lat_row[mid];
        if ((int64_t)c <= T) lo = mid + 1u; else hi = mid;
    }
    if (lo < r1 || L <= q.B - 1u) return lo;
    // positions a >= B-1: cost = floor(ceil(a/B) * lat[B] / W) + lat[B] <= T
    //   <=>  ceil(a/B) * lat[B] <= (T - lat[B] + 1) * W - 1
    const int64_t T2 = T - (int64_t)q.latB;
    if (T2 < 0) return lo;
    if (q.latB == 0u) return L;
    const uint64_t m_max = wide_div((uint64_t)(T2 + 1) * q.W - 1ull, q.latB);
    if (m_max >= (uint64_t)L) return L;
    const uint64_t a_max = m_max * q.B;                           // ceil(a/B) <= m_max  <=>  a <= m_max * B
    if (a_max + 1ull < (uint64_t)q.B) return lo;                  // below B-1: nothing of this range
    return a_max + 1ull < (uint64_t)L ? (uint32_t)(a_max + 1ull) : L;
}

// (start flag, minimum since the last start): the operator of a segmented minimum scan
__device__ __forceinline__ void seg_min_combine(uint32_t lf, int32_t lv, uint32_t& f, int32_t& v) {
    v = f ? v : (lv < v ? lv : v);
    f |= lf;
}

// inclusive segmented minimum scan across the wave
__device__ __forceinline__ void seg_min_wave_scan(uint32_t& f, int32_t& v, int lane) {
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t lf = __shfl_up(f, off);
        const int32_t lv = __shfl_up(v, off);
        if (lane >= off) seg_min_combine(lf, lv, f, v);
    }
}

__global__ __launch_bounds__(kConsTile) void consistent_prepare_kernel(SortDev A) {
    __shared__ EpiSeg tab[kEpiSegs];
    __shared__ uint32_t wave_f[kConsTile / 64];
    __shared__ int32_t wave_v[kConsTile / 64];
    const PlanDev& P = A.plan;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t segs = (int64_t)P.K * P.S;
    const bool cached = segs <= kEpiSegs;
    if (cached && tid < segs) tab[tid] = epilogue_segment(A, (uint32_t)tid);
    __syncthreads();
    const int last = ((int)A.params->passes - 1) & 1;
    uint32_t* keys = A.key[last];
    const uint32_t* pays = A.pay[last];
    int32_t* thr = reinterpret_cast<int32_t*>(A.pay[last ^ 1]);   // free since the last pass
    const uint32_t umin = ~A.params->inv_min;
    const uint32_t idx_mask = A.idx_bits >= 32 ? 0xFFFFFFFFu : ((1u << A.idx_bits) - 1u);
    const int64_t tiles = (A.n + kConsTile - 1) / kConsTile;
    const int64_t per = (tiles + A.cons_ranges - 1) / A.cons_ranges;      // this workgroup's range of tiles
    const int64_t t_lo = blockIdx.x * per < tiles ? blockIdx.x * per : tiles;
    const int64_t t_hi = t_lo + per < tiles ? t_lo + per : tiles;
    uint32_t range_f = 0;                                // thread 0: the scan's total over the range so far
    int32_t range_v = kNoMin;
    for (int64_t t = t_lo; t < t_hi; ++t) {
        const int64_t j = t * kConsTile + tid;
        const bool ok = j < A.n;
        bool can = false;
        uint32_t f = 0;
        int32_t v = kNoMin;
        if (ok) {
            const uint32_t key = keys[j], pay = pays[j];
            const uint32_t local = pay & idx_mask;
            const uint32_t seg = A.idx_bits < 32 ? (pay >> A.idx_bits) : 0u;
            EpiSeg q;
            if (cached) q = tab[seg]; else q = epilogue_segment(A, seg);
            const int32_t deadline = epilogue_deadline(A, q, key, (uint32_t)q.first + local, umin);
            keys[j] = (uint32_t)deadline;
            const unsigned long long dn = ((unsigned long long)q.down_hi << 32) | q.down_lo;
            f = j == (int64_t)q.start ? 1u : 0u;
            if (q.aux & kSegScan) {
                const int64_t rec = q.rec;
                const uint32_t i = (uint32_t)(j - (int64_t)q.start);
                const uint32_t c = deadline == kInt32Max ? (uint32_t)q.len
                                   : positions_in_time(q, P.lat + rec * PARD_LAT_ENTRIES, (int64_t)deadline - (int64_t)q.now - (int64_t)dn);
                if ((q.mode & 0xFF) == PARD_ORDER_LBF) v = (int32_t)c - (int32_t)i;
                else v = i >= c ? (int32_t)i : kNoMin;
                thr[j] = v;
            } else {
                int32_t est;
                uint8_t drp;
                finish_request((uint64_t)(q.aux & ~kSegScan) + dn, q.now, deadline, est, drp);
                can = drp == 0;
            }
        }
        const unsigned long long word = __ballot(can);
        if (lane == 0 && t * kConsTile + wave * 64 < A.n) A.alive[(t * kConsTile + wave * 64) >> 6] = word;
        // the tile's total of the segmented minimum scan
        seg_min_wave_scan(f, v, lane);
        if (lane == 63) { wave_f[wave] = f; wave_v[wave] = v; }
        __syncthreads();
        if (tid == 0) {
            uint32_t tf = wave_f[0];
            int32_t tv = wave_v[0];
            for (int w = 1; w < kConsTile / 64; ++w) {
                uint32_t wf = wave_f[w];
                int32_t wv = wave_v[w];
                seg_min_combine(tf, tv, wf, wv);
                tf = wf; tv = wv;
            }
            A.tile_tot[t] = make_uint2(range_f, (uint32_t)range_v);      // what lies before this tile inside the range
            seg_min_combine(range_f, range_v, tf, tv);
            range_f = tf; range_v = tv;
        }
        __syncthreads();
    }
    if (tid == 0) A.range_tot[blockIdx.x] = make_uint2(range_f, (uint32_t)range_v);
}

// carry[r] = minimum over the slots before range r since the last queue start: one workgroup
// scans the ranges' totals (a few per thread, then across the workgroup).
__global__ __launch_bounds__(1024) void consistent_range_scan_kernel(SortDev A) {
    __shared__ uint32_t wave_f[16];
    __shared__ int32_t wave_v[16];
    constexpr int kPer = kConsRanges / 1024;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint2 x[kPer];
#pragma unroll
    for (int i = 0; i < kPer; ++i)
        x[i] = tid * kPer + i < A.cons_ranges ? A.range_tot[tid * kPer + i] : make_uint2(0u, (uint32_t)kNoMin);
    uint32_t f = 0;
    int32_t v = kNoMin;
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        uint32_t xf = x[i].x;
        int32_t xv = (int32_t)x[i].y;
        seg_min_combine(f, v, xf, xv);
        f = xf; v = xv;
    }
    seg_min_wave_scan(f, v, lane);
    if (lane == 63) { wave_f[wave] = f; wave_v[wave] = v; }
    uint32_t ef = __shfl_up(f, 1);
    int32_t ev = __shfl_up(v, 1);
    if (lane == 0) { ef = 0u; ev = kNoMin; }
    __syncthreads();
    {
        uint32_t rf = 0u;
        int32_t rv = kNoMin;
        for (int w = 0; w < wave; ++w) {
            uint32_t wf = wave_f[w];
            int32_t wv = wave_v[w];
            seg_min_combine(rf, rv, wf, wv);
            rf = wf; rv = wv;
        }
        seg_min_combine(rf, rv, ef, ev);
    }
    int32_t run = ev;                                    // everything before this thread's ranges
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        if (tid * kPer + i < A.cons_ranges) A.carry[tid * kPer + i] = run;
        const int32_t xv = (int32_t)x[i].y;
        run = x[i].x ? xv : (run < xv ? run : xv);
    }
}

__global__ __launch_bounds__(64) void consistent_chain_kernel(SortDev A) {
    __shared__ int32_t dls[kChainWords * 64];           // deadlines of the slots of one step's words
    __shared__ unsigned long long words[kChainAhead * 64];
    const PlanDev& P = A.plan;
    const int lane = threadIdx.x;
    const uint32_t seg = blockIdx.x;
    const int64_t s0 = A.seg_ptr[seg], s1 = A.seg_ptr[seg + 1];
    if (s1 <= s0 || s1 > A.n || s0 < 0) return;
    if (A.min_lat[seg] & kSegScan) return;              // positions by prefix minimum, no walk
    const uint32_t u = seg / (uint32_t)P.S, k = seg - u * (uint32_t)P.S;
    const int64_t rec = P.shared ? (int64_t)k : (int64_t)seg;
    const StageRec sr = P.recs[rec];
    const int32_t* lat_row = P.lat + rec * PARD_LAT_ENTRIES;
    const unsigned long long dn = A.down[seg];
    const int32_t now = A.now[u];
    const int32_t* dl = reinterpret_cast<const int32_t*>(A.key[((int)A.params->passes - 1) & 1]);
    const int64_t w_first = s0 >> 6, w_last = (s1 - 1) >> 6;
    auto candidates = [&](int64_t w) -> unsigned long long {       // the queue's own bits of mask word w
        if (w > w_last) return 0ull;
        unsigned long long v = A.alive[w];
        if (w == w_first) v &= ~0ull << (s0 & 63);
        if (w == w_last && (s1 & 63)) v &= (1ull << (s1 & 63)) - 1ull;
        return v;
    };
    uint32_t kept = 0;                                  // kept requests of the queue so far (same in every lane)
    // one step settles the 64 mask words w0 .. w0+63 (lane l holds word w0 + l)
    auto step = [&](int64_t w0, unsigned long long mine) {
        const unsigned long long busy = __ballot(mine != 0ull);
        const int64_t w = w0 + lane;
        if (busy == 0ull) {                              // nobody here can be kept
            if (w <= w_last && w > w_first) A.wkept[w] = kept;
            return;
        }
        const uint32_t kept_before_step = kept;
        unsigned long long keep_mine = 0ull;
        // deadlines of the busy words into LDS, eight words' loads in flight
        for (int b0 = 0; b0 < kChainWords; b0 += 8) {
            if (((busy >> b0) & 0xFFull) == 0ull) continue;
            int32_t v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int64_t j = (w0 + b0 + i) * 64 + lane;
                v[i] = (((busy >> (b0 + i)) & 1ull) && j < A.n) ? dl[j] : 0;
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) dls[(b0 + i) * 64 + lane] = v[i];
        }
        __syncthreads();
        unsigned long long rest = busy;
        while (rest) {
            const int b = __ffsll((long long)rest) - 1;
            rest &= rest - 1ull;
            const unsigned long long m = __shfl(mine, b);
            const bool ok = (m >> lane) & 1ull;
            const int32_t deadline = dls[b * 64 + lane];
            // guess that all candidates are kept, evaluate everybody at the position the guess
            // implies, take the decisions as the next guess; a guess that reproduces itself is
            // the in-order result
            unsigned long long keep = m;
            for (int round = 0; round <= 64; ++round) {
                const uint32_t ahead = kept + __builtin_amdgcn_mbcnt_hi((uint32_t)(keep >> 32),
                                                  __builtin_amdgcn_mbcnt_lo((uint32_t)keep, 0u));
                int32_t est;
                uint8_t drp;
                finish_request(stage_cost(sr, ahead, lat_row) + dn, now, deadline, est, drp);
                const unsigned long long next = __ballot(ok && drp == 0);
                if (next == keep) break;
                keep = next;
            }
            if (lane == b) keep_mine = keep;
            kept += (uint32_t)__popcll(keep);
        }
        __syncthreads();
        // kept requests of this queue before each word of the step
        const uint32_t c = (uint32_t)__popcll(keep_mine);
        uint32_t inc = c;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t t = __shfl_up(inc, off);
            if (lane >= off) inc += t;
        }
        if (w <= w_last) {
            if (w > w_first) A.wkept[w] = kept_before_step + inc - c;
            if (keep_mine) atomicOr(&A.keepm[w], keep_mine);     // the first and last word may be shared with other queues
        }
    };
    // The mask words of kChainAhead steps are loaded at once (the next batch while this one is
    // worked on) and handed to the steps through LDS.
    unsigned long long nxt[kChainAhead];
#pragma unroll
    for (int i = 0; i < kChainAhead; ++i) nxt[i] = candidates(w_first + i * kChainWords + lane);
    for (int64_t w0 = w_first; w0 <= w_last; w0 += kChainAhead * kChainWords) {
#pragma unroll
        for (int i = 0; i < kChainAhead; ++i) words[i * 64 + lane] = nxt[i];
#pragma unroll
        for (int i = 0; i < kChainAhead; ++i) nxt[i] = candidates(w0 + (kChainAhead + i) * kChainWords + lane);
        __syncthreads();
        for (int i = 0; i < kChainAhead && w0 + i * kChainWords <= w_last; ++i) step(w0 + i * kChainWords, words[i * 64 + lane]);
        __syncthreads();
    }
}

__global__ __launch_bounds__(kConsTile) void consistent_finish_kernel(SortDev A) {
    __shared__ EpiSeg tab[kEpiSegs];
    __shared__ uint32_t wave_f[kConsTile / 64];
    __shared__ int32_t wave_v[kConsTile / 64];
    const PlanDev& P = A.plan;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t segs = (int64_t)P.K * P.S;
    const bool cached = segs <= kEpiSegs;
    if (cached && tid < segs) tab[tid] = epilogue_segment(A, (uint32_t)tid);
    __syncthreads();
    const int last = ((int)A.params->passes - 1) & 1;
    const int32_t* dl = reinterpret_cast<const int32_t*>(A.key[last]);
    const uint32_t* pays = A.pay[last];
    const int32_t* thr = reinterpret_cast<const int32_t*>(A.pay[last ^ 1]);
    uint32_t* packed = A.key[last ^ 1];
    const uint32_t idx_mask = A.idx_bits >= 32 ? 0xFFFFFFFFu : ((1u << A.idx_bits) - 1u);
    const int64_t tiles = (A.n + kConsTile - 1) / kConsTile;
    const int64_t per = (tiles + A.cons_ranges - 1) / A.cons_ranges;      // the same ranges as in the prepare kernel
    const int64_t t_lo = blockIdx.x * per < tiles ? blockIdx.x * per : tiles;
    const int64_t t_hi = t_lo + per < tiles ? t_lo + per : tiles;
    const int32_t range_carry = A.carry[blockIdx.x];
    for (int64_t t = t_lo; t < t_hi; ++t) {
        const int64_t j = t * kConsTile + tid;
        const bool ok = j < A.n;
        EpiSeg q{};
        uint32_t pay = 0, seg = 0, f = 0;
        int32_t deadline = 0, v = kNoMin;
        bool scanned = false;
        if (ok) {
            pay = pays[j];
            deadline = dl[j];
            seg = A.idx_bits < 32 ? (pay >> A.idx_bits) : 0u;
            if (cached) q = tab[seg]; else q = epilogue_segment(A, seg);
            f = j == (int64_t)q.start ? 1u : 0u;
            scanned = (q.aux & kSegScan) != 0u;
            if (scanned) v = thr[j];
        }
        // exclusive segmented minimum over the slots before j: inside the wave, the earlier waves
        // of the tile, the earlier tiles
        const uint32_t own_f = f;
        seg_min_wave_scan(f, v, lane);
        if (lane == 63) { wave_f[wave] = f; wave_v[wave] = v; }
        __syncthreads();
        uint32_t ef = __shfl_up(f, 1);
        int32_t ev = __shfl_up(v, 1);
        if (lane == 0) { ef = 0; ev = kNoMin; }
        {
            const uint2 pre = A.tile_tot[t];                   // before the tile: inside the range, and before the range
            uint32_t run_f = pre.x;
            int32_t run_v = pre.x ? (int32_t)pre.y : (range_carry < (int32_t)pre.y ? range_carry : (int32_t)pre.y);
            for (int w = 0; w < wave; ++w) {
                uint32_t wf = wave_f[w];
                int32_t wv = wave_v[w];
                seg_min_combine(run_f, run_v, wf, wv);
                run_f = wf; run_v = wv;
            }
            seg_min_combine(run_f, run_v, ef, ev);
        }
        const int32_t before = own_f ? kNoMin : ev;            // nothing lies before a queue's first slot
        __syncthreads();
        if (ok) {
            const uint32_t local = pay & idx_mask;
            const int64_t rec = q.rec;
            const uint32_t i = (uint32_t)(j - (int64_t)q.start);
            uint32_t pos;
            if (scanned) {
                if (before == kNoMin) pos = i;
                else if ((q.mode & 0xFF) == PARD_ORDER_LBF) {
                    const int64_t a = (int64_t)i - 1 + (int64_t)before;
                    pos = a < (int64_t)i ? (uint32_t)a : i;
                } else {
                    pos = (uint32_t)before < i ? (uint32_t)before : i;
                }
            } else {
                const int64_t w = j >> 6;
                const unsigned long long below = A.keepm[w] & ((1ull << (j & 63)) - 1ull);
                if (w == ((int64_t)q.start >> 6)) pos = (uint32_t)__popcll(below >> (q.start & 63));     // the queue starts inside this word
                else pos = A.wkept[w] + (uint32_t)__popcll(below);
            }
            int32_t est;
            uint8_t drp;
            finish_request(epilogue_estimate(q, P.lat + rec * PARD_LAT_ENTRIES, pos), q.now, deadline, est, drp);
            const uint32_t r = (uint32_t)q.first + local;
            A.order[j] = (int32_t)r;
            if ((int64_t)r < A.n) packed[r] = (uint32_t)est | ((uint32_t)drp << 31);
        }
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
    D.sub = a.sub;
    D.consistent = a.consistent;
    D.status_word = a.status;
    D.params = reinterpret_cast<SortParams*>(ws + L.params);
    D.seg_count = reinterpret_cast<uint32_t*>(ws + L.seg_count);
    D.cfull = reinterpret_cast<unsigned long long*>(ws + L.cfull);
    D.down = reinterpret_cast<unsigned long long*>(ws + L.down);
    D.chunk_tot = reinterpret_cast<uint32_t*>(ws + L.chunk_tot);
    D.tile_hist = reinterpret_cast<uint32_t*>(ws + L.tile_hist);
    D.chunks = L.chunks;
    D.part_minmax = reinterpret_cast<uint32_t*>(ws + L.part_minmax);
    D.part_cnt = reinterpret_cast<uint32_t*>(ws + L.part_cnt);
    D.part_flag = reinterpret_cast<uint32_t*>(ws + L.part_flag);
    D.wave_cnt = reinterpret_cast<uint32_t*>(ws + L.wave_cnt);
    for (int b = 0; b < 2; ++b) {
        D.key[b] = reinterpret_cast<uint32_t*>(ws + L.key[b]);
        D.pay[b] = reinterpret_cast<uint32_t*>(ws + L.pay[b]);
    }
    D.min_lat = reinterpret_cast<uint32_t*>(ws + L.min_lat);
    D.alive = reinterpret_cast<unsigned long long*>(ws + L.alive);
    D.keepm = reinterpret_cast<unsigned long long*>(ws + L.keepm);
    D.wkept = reinterpret_cast<uint32_t*>(ws + L.wkept);
    D.tile_tot = reinterpret_cast<uint2*>(ws + L.tile_tot);
    D.range_tot = reinterpret_cast<uint2*>(ws + L.range_tot);
    D.carry = reinterpret_cast<int32_t*>(ws + L.carry);
    D.tiles = L.tiles;
    D.idx_bits = L.idx_bits;
    D.seg_bits = L.seg_bits;
    D.max_passes = L.max_passes;
    D.ret_cursor = reinterpret_cast<uint32_t*>(ws + L.ret_cursor);
    D.ret_shift = L.ret_shift;
    D.finish_in_last_pass = (!a.consistent && L.ret_shift <= kRetMaxShift) ? 1 : 0;
    return D;
}

}  // namespace

int64_t sort_workspace_bytes(int32_t K, int32_t S, int64_t n) { return make_layout(K, S, n, n).total; }

bool sort_supported(int32_t K, int32_t S, int64_t n, int64_t max_snapshot) {
    const SortLayout L = make_layout(K, S, n, max_snapshot);
    return L.idx_bits + L.seg_bits <= 32 && n < ((int64_t)1 << 30);
}

hipError_t launch_sort_path(const SortArgs& a, hipStream_t stream) {
    const SortLayout L = make_layout(a.plan.K, a.plan.S, a.n, a.max_snapshot);
    SortDev D = make_dev(a, L);
    const int64_t zero16 = (a.consistent ? L.zero_end_consistent : L.zero_end) / 16;
    int zb = (int)((zero16 + 255) / 256);
    if (zb > 4096) zb = 4096;
    if (zb < 1) zb = 1;
    zero_kernel<<<zb, 256, 0, stream>>>(reinterpret_cast<uint4*>(a.workspace), zero16);
    int gb = (int)((a.n + 256 * 8 - 1) / (256 * 8));
    if (gb > 8192) gb = 8192;
    if (gb < 1) gb = 1;
    int sb = (int)((a.n + kChunk - 1) / kChunk);       // streaming kernels: two workgroups of 1024 threads per CU
    if (sb > 2 * a.num_cus) sb = 2 * a.num_cus;
    if (sb > kStreamBlocksMax) sb = kStreamBlocksMax;
    if (sb < 1) sb = 1;
    D.stream_blocks = sb;
    // the split below may finish the call: then the count also watches the order of the deadlines
    const bool may_split = a.n > 0 && (int64_t)a.plan.K * a.plan.S <= kPartialSegs;
    if (may_split && a.plan.uniform_mode == PARD_ORDER_LBF) count_kernel<PARD_ORDER_LBF><<<sb, kScanThreads, 0, stream>>>(D);
    else if (may_split && a.plan.uniform_mode == PARD_ORDER_HBF) count_kernel<PARD_ORDER_HBF><<<sb, kScanThreads, 0, stream>>>(D);
    else count_kernel<-1><<<sb, kScanThreads, 0, stream>>>(D);
    setup_kernel<<<1, 1024, 0, stream>>>(D);
    if (a.n > 0) {
        // finishes the call when the requests come in deadline order; everything below then finds nothing to do
        if (may_split) {
            const unsigned sg = (unsigned)(sb * kSplitPerCount);
            if (a.plan.uniform_mode == PARD_ORDER_HBF && a.consistent) split_kernel<true, true><<<sg, kSplitThreads, 0, stream>>>(D);
            else if (a.plan.uniform_mode == PARD_ORDER_HBF) split_kernel<true, false><<<sg, kSplitThreads, 0, stream>>>(D);
            else if (a.plan.uniform_mode == PARD_ORDER_LBF && a.consistent) split_kernel<false, true><<<sg, kSplitThreads, 0, stream>>>(D);
            else if (a.plan.uniform_mode == PARD_ORDER_LBF) split_kernel<false, false><<<sg, kSplitThreads, 0, stream>>>(D);
        }
        auto radix_pass = [&](auto items_tag, int p) {
            constexpr int ITEMS = decltype(items_tag)::value;
            if (p == 0) upsweep_kernel<true, ITEMS><<<(unsigned)L.tiles, kSortThreads, 0, stream>>>(D, p);
            else upsweep_kernel<false, ITEMS><<<(unsigned)L.tiles, kSortThreads, 0, stream>>>(D, p);
            if (L.chunks > kFusedScanChunks) {
                digit_scan_kernel<<<1, 1024, 0, stream>>>(D, p);
                chunk_scan_kernel<true><<<(unsigned)L.chunks, kRadix, 0, stream>>>(D, p);
            } else {
                chunk_scan_kernel<false><<<(unsigned)L.chunks, kRadix, 0, stream>>>(D, p);
            }
            const unsigned dg = (unsigned)((L.tiles + kDies - 1) / kDies * kDies);
            if (p == 0) downsweep_kernel<true, ITEMS><<<dg, kSortThreads, 0, stream>>>(D, p);
            else downsweep_kernel<false, ITEMS><<<dg, kSortThreads, 0, stream>>>(D, p);
        };
        for (int p = 0; p < L.max_passes; ++p) {
            if (L.tile_items == kSmallItems) radix_pass(std::integral_constant<int, kSmallItems>{}, p);
            else radix_pass(std::integral_constant<int, kSortItems>{}, p);
        }
        if (a.consistent) {
            int64_t pg = (a.n + kConsTile - 1) / kConsTile;
            if (pg > 16 * (int64_t)a.num_cus) pg = 16 * (int64_t)a.num_cus;
            if (pg > kConsRanges) pg = kConsRanges;
            D.cons_ranges = (int32_t)pg;
            consistent_prepare_kernel<<<(unsigned)pg, kConsTile, 0, stream>>>(D);
            consistent_range_scan_kernel<<<1, 1024, 0, stream>>>(D);
            consistent_chain_kernel<<<(unsigned)((int64_t)a.plan.K * a.plan.S), 64, 0, stream>>>(D);
            consistent_finish_kernel<<<(unsigned)pg, kConsTile, 0, stream>>>(D);
        } else {
            int64_t eg = (a.n / 4 + kEpiThreads - 1) / kEpiThreads;       // persistent: a few workgroups per compute unit
            if (eg > 8 * (int64_t)a.num_cus) eg = 8 * (int64_t)a.num_cus;
            if (eg < 1) eg = 1;
            if (!D.finish_in_last_pass) {
                // more requests than kRetBuckets ranges of the largest size hold (2^25): results go back one by one
                epilogue_kernel<<<(unsigned)eg, kEpiThreads, 0, stream>>>(D);
                unpack_kernel<<<gb, 256, 0, stream>>>(D);
            } else {
                const unsigned ranges = (unsigned)((a.n + ((int64_t)1 << L.ret_shift) - 1) >> L.ret_shift);
                switch (L.ret_shift) {
                    case 11: epilogue_return_kernel<11, 256><<<ranges, 256, 0, stream>>>(D); break;
                    case 12: epilogue_return_kernel<12, 256><<<ranges, 256, 0, stream>>>(D); break;
                    case 13: epilogue_return_kernel<13, 512><<<ranges, 512, 0, stream>>>(D); break;
                    case 14: epilogue_return_kernel<14, 1024><<<ranges, 1024, 0, stream>>>(D); break;
                    default: epilogue_return_kernel<15, 1024><<<ranges, 1024, 0, stream>>>(D); break;
                }
            }
        }
        if (a.consistent) unpack_kernel<<<gb, 256, 0, stream>>>(D);
    }
    return hipGetLastError();
}

}  // namespace pard
