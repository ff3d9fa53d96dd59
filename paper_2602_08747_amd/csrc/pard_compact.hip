// Drop-mask stream compaction: the survivor queues (paper Section 4.1: the Request Broker
// keeps or drops each request; the kept ones, in queue order, form the next batches).
//
// keep[j] = !drop[order[j]] for every queue slot j; surv_idx is order filtered by keep;
// surv_ptr[g] = number of kept slots before queue g starts.
//
// Two paths.  Snapshots that fit one workgroup are compacted one per workgroup (second half of this
// file).  Anything larger is compacted as one stream of tiles of 4096 queue slots in three steps, none of
// which waits for another workgroup:
//   count   every tile looks its slots' decisions up and leaves the keep flags by slot (four to a byte) and
//           its number of kept slots
//   (scan)  beyond 4096 tiles one workgroup turns the counts into offsets; up to there every workgroup of
//           the last step adds up the counts before its tile itself
//   write   every tile reads its keep flags, loads the request ids of the groups of four slots that keep
//           somebody, and writes its survivors as one contiguous run, together with the offsets of the queues
//           that start inside it.
// (An earlier one-pass form, in which persistent workgroups published their counts and a scan wave handed out
// the offsets, needed every workgroup resident at once to be sure that its bounded waits end; this form costs
// a second read of the kept slots' ids and nothing else: 16.8 million slots 45 -> 41 us, 8.4 million in
// snapshots of 64 requests 42 -> 32 us, 33.5 million in snapshots of 1024 88 -> 95 us.)
#include <type_traits>

#include "pard_device.hpp"

namespace pard {

namespace {

constexpr int kCThreads = 256;
constexpr int kCItems = 16;
constexpr int kCTile = kCThreads * kCItems;            // 4096 queue slots per tile
constexpr int kCWaves = kCThreads / kWave;
constexpr int kStageLds = 2 * kCTile + 256;            // bytes of LDS that stage a tile's slice of drop[]
constexpr int kStageBytes = kStageLds - 32;            // widest request-id range staged in LDS
constexpr int kStageChunks = (kStageLds / 16 + kCThreads - 1) / kCThreads;   // 16-byte chunks per thread

// What a tile needs to know before it has seen its slots.
struct TileInfo {
    int32_t id_lo;      // the ids in the tile's slots lie in [id_lo, id_lo + id_span) ...
    int32_t id_span;    // ... or 0 when that range is unknown or too wide to stage
    int32_t g0, g1;     // queues g0 <= g < g1 start in this tile (their offsets are its to write)
};

// Queue g = u * S + s holds requests of snapshot u only, and the requests of snapshot u are
// the ids [seg_ptr[u*S], seg_ptr[(u+1)*S]) (snapshots are contiguous in the request arrays
// and their queues contiguous in queue order), so the snapshots a tile overlaps bound its
// ids.  The bound is only a hint: a slot whose id falls outside it is looked up by request id
// instead.
//
// Lookups by request id: from the byte array such a lookup fetches a whole memory sector per byte (16.8
// million shuffled ids: 1 GB for 16.8 MB of decisions), so when the promised snapshot bound is above what a
// tile can stage, the decisions are first packed into keep bits (bit r of the array: request r is kept; 2 MB
// for as many requests, which stay in the L2) and the lookups read those.

// 16 queue slots per thread: wave w owns slots [w*1024, (w+1)*1024) of the tile, load k covers
// 256 of them, 4 consecutive slots per lane.  Slots past the end of the data read as -1.
__device__ __forceinline__ void load_tile_ids(const CompactArgs& A, int64_t base, int valid, bool vec, int wave, int lane,
                                              int32_t (&ids)[4][4]) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int e = wave * 1024 + k * 256 + lane * 4;
        if (vec && e + 3 < valid) {
            const int4 v = *reinterpret_cast<const int4*>(A.order + base + e);
            ids[k][0] = v.x; ids[k][1] = v.y; ids[k][2] = v.z; ids[k][3] = v.w;
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c) ids[k][c] = e + c < valid ? A.order[base + e + c] : -1;
        }
    }
}

// No requests: every queue offset is zero.
__global__ void compact_empty_kernel(int32_t* surv_ptr, int32_t num_segments) {
    for (int g = blockIdx.x * blockDim.x + threadIdx.x; g <= num_segments; g += gridDim.x * blockDim.x) surv_ptr[g] = 0;
}

// ---- the stream of tiles: count, (scan), write ------------------------------------------------------------
// Smallest g in [0, count] with seg_ptr[g] >= x (count when there is none); seg_ptr never falls.  All 64 lanes of a
// wave call this with the same arguments: every round they probe 64 evenly spaced entries at once.
__device__ __forceinline__ int first_at_least_wave(const int32_t* seg_ptr, int count, int64_t x, int lane) {
    int lo = 0, hi = count;                      // entries before lo are below x, entries from hi on are not
    while (lo < hi) {
        const int step = (hi - lo + kWave - 1) / kWave;
        const int probe = lo + (lane + 1) * step - 1;
        const bool below = probe < hi && (int64_t)seg_ptr[probe] < x;
        const int cnt = __popcll(__ballot(below));          // these lanes are a prefix
        const int old = lo;
        lo = old + cnt * step;
        const int stop = old + (cnt + 1) * step - 1;        // the first probe that was not below x
        if (stop < hi) hi = stop;
        if (lo > hi) lo = hi;
    }
    return lo;
}

// TileInfo of tile t, computed by a wave.
__device__ __forceinline__ TileInfo tile_info_wave(const int32_t* seg_ptr, int32_t num_segments, int32_t stages, int64_t n,
                                                   int64_t t, int64_t tiles, int lane) {
    const int64_t ta = t * kCTile, tb = ta + kCTile;
    const int la = first_at_least_wave(seg_ptr, num_segments + 1, ta, lane);
    const int lb = first_at_least_wave(seg_ptr, num_segments + 1, tb, lane);
    TileInfo ti;
    ti.g0 = la;
    ti.g1 = t + 1 == tiles ? num_segments + 1 : lb;           // the last tile also takes offsets equal to n
    int32_t x = (la <= num_segments && (int64_t)seg_ptr[la] == ta) ? la : la - 1;
    int32_t y = lb - 1;
    x = x < 0 ? 0 : (x > num_segments - 1 ? num_segments - 1 : x);
    y = y < 0 ? 0 : (y > num_segments - 1 ? num_segments - 1 : y);
    const int64_t lo = seg_ptr[(x / stages) * stages], hi = seg_ptr[(y / stages + 1) * stages];
    const bool ok = lo >= 0 && hi > lo && hi <= n && hi - lo <= kStageBytes;
    ti.id_lo = ok ? (int32_t)lo : 0;
    ti.id_span = ok ? (int32_t)(hi - lo) : 0;
    return ti;
}

// Packs the decisions into keep bits.
__global__ void compact_pack_kernel(const uint8_t* drop, int64_t n, uint32_t* keep_bits) {
    const bool vec = (reinterpret_cast<uintptr_t>(drop) & 15) == 0;
    const int64_t nwords = (n + 31) / 32;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; w < nwords; w += stride) {
        const int64_t r0 = w * 32;
        uint32_t bits = 0;
        if (vec && r0 + 31 < n) {
            const uint4 a = *reinterpret_cast<const uint4*>(drop + r0), b = *reinterpret_cast<const uint4*>(drop + r0 + 16);
            const uint32_t v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
            for (int q = 0; q < 8; ++q)
#pragma unroll
                for (int c = 0; c < 4; ++c) bits |= (uint32_t)(((v[q] >> (8 * c)) & 0xFFu) == 0u) << (4 * q + c);
        } else {
            for (int c = 0; c < 32; ++c)
                if (r0 + c < n && drop[r0 + c] == 0) bits |= 1u << c;
        }
        keep_bits[w] = bits;
    }
}

// First kernel: the keep flags of every slot of a tile (four to a byte, laid out as the loads of load_tile_ids are)
// and the tile's number of kept slots.
__global__ __launch_bounds__(kCThreads) void compact_count_kernel(CompactArgs A, TileInfo* info, uint32_t* tile_count,
                                                                  uint8_t* slot_keep, const uint32_t* keep_bits, int64_t tiles) {
    __shared__ __align__(16) uint8_t drop_l[kStageLds];
    __shared__ uint32_t wave_tot[kCWaves];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t tile = blockIdx.x;
    const TileInfo ti = tile_info_wave(A.seg_ptr, A.num_segments, A.stages, A.n, tile, tiles, lane);
    if (tid == 0) info[tile] = ti;
    const bool vec = (reinterpret_cast<uintptr_t>(A.order) & 15) == 0;
    const uintptr_t drop_addr = reinterpret_cast<uintptr_t>(A.drop);
    const uintptr_t end_addr = drop_addr + (uintptr_t)A.n;
    const int64_t base = tile * kCTile;
    const int64_t left = A.n - base;
    const int valid = (int)(left < kCTile ? left : kCTile);
    int32_t ids[4][4];
    load_tile_ids(A, base, valid, vec, wave, lane, ids);
    const bool staged = ti.id_span > 0;
    uint32_t delta = 0;
    if (staged) {
        // 16-byte chunks at 16-byte aligned addresses from just below drop[id_lo]
        const uintptr_t win = (drop_addr + (uint32_t)ti.id_lo) & ~(uintptr_t)15;
        delta = (uint32_t)(drop_addr + (uint32_t)ti.id_lo - win);              // 0..15
        const uint32_t chunks = (delta + (uint32_t)ti.id_span + 15u) >> 4;      // <= kStageLds / 16
        uint4 chunk[kStageChunks];
#pragma unroll
        for (int q = 0; q < kStageChunks; ++q) {
            const uint32_t c = (uint32_t)(q * kCThreads + tid);
            const uintptr_t a = win + 16u * (uintptr_t)c;
            uint4 v = make_uint4(0x01010101u, 0x01010101u, 0x01010101u, 0x01010101u);
            if (c < chunks) {
                if (a >= drop_addr && a + 16 <= end_addr) {
                    v = *reinterpret_cast<const uint4*>(a);
                } else {                                         // chunk straddles an end of the array
                    uint32_t w[4] = {v.x, v.y, v.z, v.w};
                    for (int b = 0; b < 16; ++b) {
                        const uintptr_t ab = a + b;
                        if (ab >= drop_addr && ab < end_addr) {
                            const uint32_t byte = *reinterpret_cast<const uint8_t*>(ab);
                            w[b >> 2] = (w[b >> 2] & ~(0xFFu << (8 * (b & 3)))) | (byte << (8 * (b & 3)));
                        }
                    }
                    v = make_uint4(w[0], w[1], w[2], w[3]);
                }
            }
            chunk[q] = v;
        }
#pragma unroll
        for (int q = 0; q < kStageChunks; ++q) {
            const uint32_t c = (uint32_t)(q * kCThreads + tid);
            if (c < chunks) *reinterpret_cast<uint4*>(drop_l + 16u * c) = chunk[q];
        }
    }
    __syncthreads();
    uint32_t keep[4];
    bool slow = !staged;                // some slot of this thread needs a lookup by request id
    if (staged) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            keep[k] = 0;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t d = (uint32_t)ids[k][c] - (uint32_t)ti.id_lo;
                const bool in = d < (uint32_t)ti.id_span;
                const uint32_t byte = drop_l[delta + (in ? d : 0u)];
                keep[k] |= (uint32_t)(in && byte == 0) << c;
                slow |= !in;
            }
        }
    }
    if (slow) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            keep[k] = 0;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t r = (uint32_t)ids[k][c];
                if ((int64_t)r < A.n) {
                    if (keep_bits) keep[k] |= ((keep_bits[r >> 5] >> (r & 31u)) & 1u) << c;
                    else if (A.drop[r] == 0) keep[k] |= 1u << c;
                }
            }
        }
    }
    uint32_t cnt = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        slot_keep[tile * (kCTile / 4) + wave * 256 + k * 64 + lane] = (uint8_t)keep[k];
        cnt += (uint32_t)__popc(keep[k]);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) cnt += __shfl_xor(cnt, off);
    if (lane == 0) wave_tot[wave] = cnt;
    __syncthreads();
    if (tid == 0) {
        uint32_t total = 0;
        for (int w = 0; w < kCWaves; ++w) total += wave_tot[w];
        tile_count[tile] = total;
    }
}

// Exclusive scan of the tile counts by one workgroup (only for more tiles than a workgroup of the writing kernel
// adds up by itself).
__global__ __launch_bounds__(1024) void compact_tile_scan_kernel(const uint32_t* tile_count, int64_t tiles, uint32_t* tile_off) {
    __shared__ uint32_t wave_tot[16];
    __shared__ uint32_t carry;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) carry = 0;
    __syncthreads();
    for (int64_t b = 0; b < tiles; b += 1024 * 8) {
        uint32_t v[8], sum = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) { const int64_t t = b + (int64_t)tid * 8 + i; v[i] = t < tiles ? tile_count[t] : 0u; sum += v[i]; }
        uint32_t inc = sum;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) { const uint32_t x = __shfl_up(inc, off); if (lane >= off) inc += x; }
        if (lane == 63) wave_tot[wave] = inc;
        __syncthreads();
        uint32_t run = carry + inc - sum;
        for (int w = 0; w < wave; ++w) run += wave_tot[w];
#pragma unroll
        for (int i = 0; i < 8; ++i) { const int64_t t = b + (int64_t)tid * 8 + i; if (t < tiles) tile_off[t] = run; run += v[i]; }
        __syncthreads();
        if (tid == 1023) carry = run;
        __syncthreads();
    }
}

// Last kernel: a tile's survivors leave as one contiguous run at the number of kept slots in the tiles before it,
// together with the offsets of the queues that start inside it.  Slots that were dropped are not even loaded.
constexpr int kSelfSumTiles = kCThreads * 16;          // up to here a workgroup adds up the counts before its tile itself
__global__ __launch_bounds__(kCThreads) void compact_write_kernel(CompactArgs A, const TileInfo* info, const uint32_t* tile_count,
                                                                  const uint32_t* tile_off, const uint8_t* slot_keep) {
    __shared__ int32_t surv[kCTile + kWave];           // + one dump word per lane
    __shared__ uint32_t group[kCTile / 4];             // per group of 4 slots: kept slots of the tile before it | keep bits << 13
    __shared__ uint32_t wave_tot[kCWaves];
    __shared__ uint32_t wave_sum[kCWaves];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t tile = blockIdx.x;
    const int64_t base = tile * kCTile;
    const int64_t left = A.n - base;
    const int valid = (int)(left < kCTile ? left : kCTile);
    const bool vec = (reinterpret_cast<uintptr_t>(A.order) & 15) == 0;
    // kept slots in the tiles before this one
    uint32_t before_me = 0;
    if (tile_off) {
        before_me = tile_off[tile];
    } else {
        uint32_t part[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) { const int64_t t = (int64_t)i * kCThreads + tid; part[i] = t < tile ? tile_count[t] : 0u; }
#pragma unroll
        for (int i = 0; i < 16; ++i) before_me += part[i];
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) before_me += __shfl_xor(before_me, off);
        if (lane == 0) wave_sum[wave] = before_me;
    }
    uint32_t keep[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) keep[k] = slot_keep[tile * (kCTile / 4) + wave * 256 + k * 64 + lane];
    // the ids of the groups with a kept slot
    int32_t ids[4][4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int e = wave * 1024 + k * 256 + lane * 4;
#pragma unroll
        for (int c = 0; c < 4; ++c) ids[k][c] = -1;
        if (keep[k]) {
            if (vec && e + 3 < valid) {
                const int4 v = *reinterpret_cast<const int4*>(A.order + base + e);
                ids[k][0] = v.x; ids[k][1] = v.y; ids[k][2] = v.z; ids[k][3] = v.w;
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c) ids[k][c] = e + c < valid ? A.order[base + e + c] : -1;
            }
        }
    }
    // Kept slots before each of this lane's four groups inside the wave's 1024 slots: one scan for all four loads,
    // their counts packed into bytes.  The scan runs over the counts shifted up by one lane, so every partial sum
    // is an exclusive count (<= 252 fits a byte).
    const uint32_t cnt = (uint32_t)__popc(keep[0]) | ((uint32_t)__popc(keep[1]) << 8) |
                         ((uint32_t)__popc(keep[2]) << 16) | ((uint32_t)__popc(keep[3]) << 24);
    uint32_t exc = __shfl_up(cnt, 1);
    if (lane == 0) exc = 0;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t t = __shfl_up(exc, off);
        if (lane >= off) exc += t;
    }
    const uint32_t e63 = (uint32_t)__builtin_amdgcn_readlane((int)exc, 63), c63 = (uint32_t)__builtin_amdgcn_readlane((int)cnt, 63);
    uint32_t load_before[4], wave_total = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        load_before[k] = wave_total;
        wave_total += ((e63 >> (8 * k)) & 0xFFu) + ((c63 >> (8 * k)) & 0xFFu);
    }
    if (lane == 0) wave_tot[wave] = wave_total;
    __syncthreads();
    uint32_t wave_before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kCWaves; ++w) {
        const uint32_t t = wave_tot[w];
        if (w < wave) wave_before += t;
        total += t;
    }
    if (!tile_off) {
        before_me = 0;
#pragma unroll
        for (int w = 0; w < kCWaves; ++w) before_me += wave_sum[w];
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t o = wave_before + load_before[k] + ((exc >> (8 * k)) & 0xFFu);
        group[wave * 256 + k * 64 + lane] = o | (keep[k] << 13);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const bool kept = (keep[k] >> c) & 1u;
            const uint32_t at = kept ? o + (uint32_t)__popc(keep[k] & ((1u << c) - 1u)) : (uint32_t)(kCTile + lane);
            surv[at] = ids[k][c];
        }
    }
    __syncthreads();
    for (uint32_t j = tid; j < total; j += kCThreads) A.surv_idx[before_me + j] = surv[j];
    const TileInfo ti = info[tile];
    for (int32_t g = ti.g0 + tid; g < ti.g1; g += kCThreads) {
        int64_t p = (int64_t)A.seg_ptr[g] - base;
        if (p < 0) p = 0;
        uint32_t before = total;
        if (p < valid) {
            const uint32_t v = group[p >> 2];
            before = (v & 0x1FFFu) + (uint32_t)__popc((v >> 13) & ((1u << (p & 3)) - 1u));
        }
        A.surv_ptr[g] = (int32_t)(before_me + before);
    }
}

// =====================================================================================
// Snapshots that fit one workgroup (at most kLCap queue slots each): no offset chain at all.
//
// The queue slots of snapshot u, [seg_ptr[u*S], seg_ptr[(u+1)*S]), hold exactly the request
// ids of the same range (snapshots are contiguous in the request arrays and order[] permutes
// inside a snapshot), so the number of survivors of a snapshot is the number of zero bytes
// in that range of drop[] - a contiguous read that needs neither order[] nor a scan over
// tiles.  A first kernel counts them per snapshot; the main kernel gives every snapshot to
// one workgroup, which adds up the counts of the snapshots before it and then works alone.
// =====================================================================================
// The workgroup has THREADS threads and handles up to 16 * THREADS queue slots; the launcher picks
// the smaller of the two that covers the promised snapshot bound.  Below kLocalMin requests per
// snapshot a workgroup's fixed costs (and, further down, the sheer number of workgroups) outweigh what
// the missing offset chain saves, and the chained compaction above, whose cost depends on the
// number of queue slots alone, is the faster one: measured on 33.5 M requests it takes 0.08 ms at
// every snapshot size, the per-snapshot form 0.05 ms at 8192 requests per snapshot, 0.06 at 4096,
// 0.09 at 2048 and 0.14 at 1024.
constexpr int kLThreadsMax = 512;
constexpr int kLCap = kLThreadsMax * 16;               // queue slots the largest workgroup handles
constexpr int kLocalMin = 2048;                        // promised bounds up to here take the chained form
static_assert(kLCap == PARD_FUSED_SNAPSHOT_CAPACITY, "per-snapshot compaction covers the on-chip snapshot size");

// number of zero bytes in a word
__device__ __forceinline__ uint32_t zero_bytes(uint32_t w) {
    const uint32_t t = (w & 0x7F7F7F7Fu) + 0x7F7F7F7Fu;         // bit 7 of a byte: its low 7 bits are not all zero
    return (uint32_t)__popc(~(t | w | 0x7F7F7F7Fu));             // bit 7 set only where the whole byte is zero
}

// Slot range of snapshot u; false when it breaks the promised bound or the array limits.
__device__ __forceinline__ bool snapshot_range(const int32_t* seg_ptr, int64_t u, int32_t stages, int64_t n, int64_t cap,
                                               int64_t& a, int64_t& b) {
    a = seg_ptr[u * stages];
    b = seg_ptr[(u + 1) * stages];
    return a >= 0 && b >= a && b <= n && b - a <= cap;
}

template <int THREADS>
__global__ __launch_bounds__(THREADS) void snapshot_kept_kernel(const int32_t* seg_ptr, int32_t stages, int64_t n, int64_t cap,
                                                                const uint8_t* drop, uint32_t* kept, uint32_t* status_word) {
    __shared__ uint32_t part[THREADS / kWave];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t u = blockIdx.x;
    int64_t a, b;
    if (!snapshot_range(seg_ptr, u, stages, n, cap, a, b)) {
        if (tid == 0) { atomicOr(status_word, kStatusSnapshotTooLarge); kept[u] = 0; }
        return;
    }
    const uintptr_t lo = reinterpret_cast<uintptr_t>(drop) + (uintptr_t)a, hi = reinterpret_cast<uintptr_t>(drop) + (uintptr_t)b;
    const uintptr_t win = lo & ~(uintptr_t)15;
    const uint32_t chunks = (uint32_t)((hi - win + 15) >> 4);
    uint32_t cnt = 0;
    for (uint32_t c = tid; c < chunks; c += THREADS) {
        const uintptr_t at = win + 16u * (uintptr_t)c;
        if (at >= lo && at + 16 <= hi) {
            const uint4 v = *reinterpret_cast<const uint4*>(at);
            cnt += zero_bytes(v.x) + zero_bytes(v.y) + zero_bytes(v.z) + zero_bytes(v.w);
        } else {
            for (int i = 0; i < 16; ++i)
                if (at + i >= lo && at + i < hi) cnt += *reinterpret_cast<const uint8_t*>(at + i) == 0 ? 1u : 0u;
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) cnt += __shfl_xor(cnt, off);
    if (lane == 0) part[wave] = cnt;
    __syncthreads();
    if (tid == 0) {
        uint32_t sum = 0;
        for (int w = 0; w < THREADS / kWave; ++w) sum += part[w];
        kept[u] = sum;
    }
}

// Exclusive scan of kept[0..count) by one workgroup (only for very many snapshots).
__global__ __launch_bounds__(1024) void snapshot_offsets_kernel(const uint32_t* kept, int64_t count, uint32_t* snap_off) {
    __shared__ uint32_t wave_tot[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t per = (count + 1023) / 1024;
    const int64_t lo = tid * per, hi = lo + per < count ? lo + per : count;
    uint32_t sum = 0;
    for (int64_t i = lo; i < hi; ++i) sum += kept[i];
    uint32_t inc = sum;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t t = __shfl_up(inc, off);
        if (lane >= off) inc += t;
    }
    if (lane == 63) wave_tot[wave] = inc;
    __syncthreads();
    uint32_t run = inc - sum;
    for (int w = 0; w < wave; ++w) run += wave_tot[w];
    for (int64_t i = lo; i < hi; ++i) { snap_off[i] = run; run += kept[i]; }
}

template <int THREADS>
struct LocalLds {
    uint32_t group[THREADS * 4];        // per group of 4 slots: kept slots of the snapshot before it | keep bits << 13
    __align__(16) uint8_t drop[THREADS * 16 + 32];
    uint32_t wave_tot[THREADS / kWave];
    uint32_t wave_off[THREADS / kWave];
};

template <int THREADS>
__global__ __launch_bounds__(THREADS, 4) void compact_local_kernel(CompactArgs A, const uint32_t* kept, const uint32_t* snap_off) {
    constexpr int kLThreads = THREADS, kLWaves = THREADS / kWave;
    __shared__ LocalLds<THREADS> L;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t u = blockIdx.x;
    const uint32_t my_kept = kept[u];   // asked for together with the snapshot's bounds: what is loaded below depends on both
    int64_t a, b;
    if (!snapshot_range(A.seg_ptr, u, A.stages, A.n, (int64_t)THREADS * 16, a, b)) return;     // reported by the counting kernel
    const int size = (int)(b - a);
    // a snapshot without survivors (its slice of drop[] has no zero byte) only owes its queue offsets:
    // neither its slots nor its drop bytes are read
    const int load_size = my_kept == 0 ? 0 : size;

    // this snapshot's slots: wave w owns [w*1024, (w+1)*1024), load k covers 256 of them, 4 per lane.
    // Slot q of the snapshot is element q + off of that layout, off = a mod 4 when order[] allows 16-byte
    // loads, so that a lane's four slots sit on a 16-byte boundary whatever the snapshot's first slot is
    // (the off elements before the snapshot are masked out).
    const int shift = (int)(a & 3);
    const int off = ((reinterpret_cast<uintptr_t>(A.order) & 15) == 0 && size + shift <= kLThreads * 16) ? shift : 0;
    const int32_t* slots = A.order + a - off;
    const bool vec = (reinterpret_cast<uintptr_t>(slots) & 15) == 0;
    int32_t ids[4][4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int e = wave * 1024 + k * 256 + lane * 4;
        if (vec && e + 3 < load_size + off) {
            const int4 v = *reinterpret_cast<const int4*>(slots + e);
            ids[k][0] = e + 0 >= off ? v.x : -1; ids[k][1] = e + 1 >= off ? v.y : -1;
            ids[k][2] = e + 2 >= off ? v.z : -1; ids[k][3] = v.w;
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c) ids[k][c] = (e + c >= off && e + c < load_size + off) ? slots[e + c] : -1;
        }
    }
    // its slice of drop[]: 16-byte chunks at 16-byte aligned addresses from just below drop[a]
    const uintptr_t lo = reinterpret_cast<uintptr_t>(A.drop) + (uintptr_t)a, hi = reinterpret_cast<uintptr_t>(A.drop) + (uintptr_t)b;
    const uintptr_t win = lo & ~(uintptr_t)15;
    const uint32_t delta = (uint32_t)(lo - win);
    const uint32_t chunks = load_size ? (uint32_t)((hi - win + 15) >> 4) : 0u;   // <= kLCap / 16 + 2
    for (uint32_t c = tid; c < chunks; c += kLThreads) {
        const uintptr_t at = win + 16u * (uintptr_t)c;
        uint4 v;
        if (at >= lo && at + 16 <= hi) {
            v = *reinterpret_cast<const uint4*>(at);
        } else {
            uint32_t w[4] = {0x01010101u, 0x01010101u, 0x01010101u, 0x01010101u};
            for (int i = 0; i < 16; ++i)
                if (at + i >= lo && at + i < hi) {
                    const uint32_t byte = *reinterpret_cast<const uint8_t*>(at + i);
                    w[i >> 2] = (w[i >> 2] & ~(0xFFu << (8 * (i & 3)))) | (byte << (8 * (i & 3)));
                }
            v = make_uint4(w[0], w[1], w[2], w[3]);
        }
        *reinterpret_cast<uint4*>(L.drop + 16u * c) = v;
    }
    // the offsets of this snapshot's queues (the last snapshot also owns the end offset), fetched early
    const int owned = A.stages + (u + 1 == gridDim.x ? 1 : 0);
    static_assert(PARD_MAX_STAGES + 1 <= 2 * kLThreads, "at most two queue offsets per thread");
    const int64_t my_slot = tid < owned ? (int64_t)A.seg_ptr[u * A.stages + tid] - a : 0;
    // survivors of the snapshots before this one
    uint32_t before_me = 0;
    if (snap_off) {
        before_me = tid == 0 ? snap_off[u] : 0u;
    } else {
        uint32_t x[16];                 // sixteen counts per thread (the launcher scans first when there are more): all loads in flight at once
#pragma unroll
        for (int i = 0; i < 16; ++i) x[i] = (int64_t)(tid + i * kLThreads) < u ? kept[tid + i * kLThreads] : 0u;
#pragma unroll
        for (int i = 0; i < 16; ++i) before_me += x[i];
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) before_me += __shfl_xor(before_me, off);
    if (lane == 0) L.wave_off[wave] = before_me;
    __syncthreads();

    uint32_t keep[4];
    bool slow = false;                  // an id outside the snapshot's range: look it up in global memory
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        keep[k] = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint32_t d = (uint32_t)ids[k][c] - (uint32_t)a;
            const bool in = d < (uint32_t)size;
            const uint32_t byte = L.drop[delta + (in ? d : 0u)];
            keep[k] |= (uint32_t)(in && byte == 0) << c;
            slow |= !in && ids[k][c] != -1;
        }
    }
    if (slow) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            keep[k] = 0;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t r = (uint32_t)ids[k][c];
                if ((int64_t)r < A.n && A.drop[r] == 0) keep[k] |= 1u << c;
            }
        }
    }
    // one scan for all four loads: counts packed into bytes, shifted up one lane so that every
    // partial sum is an exclusive count (<= 252)
    const uint32_t cnt = (uint32_t)__popc(keep[0]) | ((uint32_t)__popc(keep[1]) << 8) |
                         ((uint32_t)__popc(keep[2]) << 16) | ((uint32_t)__popc(keep[3]) << 24);
    uint32_t exc = __shfl_up(cnt, 1);
    if (lane == 0) exc = 0;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t t = __shfl_up(exc, off);
        if (lane >= off) exc += t;
    }
    const uint32_t e63 = (uint32_t)__builtin_amdgcn_readlane((int)exc, 63), c63 = (uint32_t)__builtin_amdgcn_readlane((int)cnt, 63);
    uint32_t load_before[4], wave_total = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        load_before[k] = wave_total;
        wave_total += ((e63 >> (8 * k)) & 0xFFu) + ((c63 >> (8 * k)) & 0xFFu);
    }
    if (lane == 0) L.wave_tot[wave] = wave_total;
    __syncthreads();
    uint32_t wave_before = 0, total = 0, off0 = 0;
#pragma unroll
    for (int w = 0; w < kLWaves; ++w) {
        const uint32_t t = L.wave_tot[w];
        if (w < wave) wave_before += t;
        total += t;
        off0 += L.wave_off[w];
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        uint32_t o = wave_before + load_before[k] + ((exc >> (8 * k)) & 0xFFu);
        L.group[wave * 256 + k * 64 + lane] = o | (keep[k] << 13);
        o += off0;
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (keep[k] & (1u << c)) { A.surv_idx[o] = ids[k][c]; ++o; }
    }
    __syncthreads();
    for (int q = tid; q < owned; q += kLThreads) {          // the smallest workgroup may own more offsets than it has threads
        const int64_t slot = q == tid ? my_slot : (int64_t)A.seg_ptr[u * A.stages + q] - a;
        const int64_t p = slot < 0 ? 0 : slot;
        uint32_t before = total;
        if (p < size) {
            const int64_t ps = p + off;                  // the slot's place in the shifted layout
            const uint32_t v = L.group[ps >> 2];
            before = (v & 0x1FFFu) + (uint32_t)__popc((v >> 13) & ((1u << (ps & 3)) - 1u));
        }
        A.surv_ptr[u * A.stages + q] = (int32_t)(off0 + before);
    }
}

// After an estimate call that staged every snapshot's survivors (in queue order, from the snapshot's first
// request's place on) and a scan of the per-snapshot counts: one wave per snapshot moves its survivors and queue
// offsets to their final place.  Everything a wave needs first comes from one round of independent loads, the
// survivors from a second one.  (Measured alternatives for 4096 snapshots: every wave adding up all earlier
// counts itself 22 us - all waves of the device read the same few cache lines at once; 64 workgroups that add
// them up once and move 64 snapshots each 52 us - too few, too long chains of dependent loads.)
__global__ __launch_bounds__(kWave) void move_staged_kernel(CompactArgs A, const uint32_t* snap_off) {
    const int lane = threadIdx.x;
    const int64_t u = blockIdx.x, K = A.num_segments / A.stages;
    const int64_t a = A.seg_ptr[u * A.stages], b = A.seg_ptr[(u + 1) * A.stages];
    const uint32_t mine = A.kept[u], first = snap_off[u];
    const uint32_t loc = lane < A.stages ? (uint32_t)A.loc_ptr[u * A.stages + lane] : 0u;
    if (a < 0 || b > A.n || b - a < (int64_t)mine || b - a > (int64_t)PARD_FUSED_SNAPSHOT_CAPACITY ||
        (int64_t)first + mine > A.n) return;                                            // only after a broken promise
    const int32_t* __restrict__ src = A.staged + a + staging_shift(u, (uint32_t)(b - a), mine);
    int32_t* __restrict__ dst = A.surv_idx;
    for (uint32_t i0 = 0; i0 < mine; i0 += 16 * kWave) {
        int32_t v[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = i0 + i * kWave + lane < mine ? __builtin_nontemporal_load(src + i0 + i * kWave + lane) : 0;
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if (i0 + i * kWave + lane < mine) __builtin_nontemporal_store(v[i], dst + first + i0 + i * kWave + lane);
    }
    if (lane < A.stages) A.surv_ptr[u * A.stages + lane] = (int32_t)(first + loc);
    if (u + 1 == K && lane == 0) A.surv_ptr[K * A.stages] = (int32_t)(first + mine);
}

}  // namespace

bool compact_per_snapshot(int64_t max_snapshot) { return max_snapshot > kLocalMin && max_snapshot <= kLCap; }

int64_t compact_workspace_bytes(int64_t n, int64_t num_snapshots) {
    const int64_t tiles = (n + kCTile - 1) / kCTile;
    const int64_t chain = 2 * (((tiles + 1) * 4 + 255) & ~(int64_t)255) +                // tile counts, tile offsets
                          (((tiles + 1) * (int64_t)sizeof(TileInfo) + 255) & ~(int64_t)255) +
                          (((n + 31) / 32 * 4 + 255) & ~(int64_t)255) +                  // one keep bit per request
                          (((tiles * (kCTile / 4)) + 255) & ~(int64_t)255);              // keep flags by queue slot, four to a byte
    const int64_t local = 2 * ((num_snapshots * 4 + 255) & ~(int64_t)255);
    return chain > local ? chain : local;
}

hipError_t launch_compact(const CompactArgs& a, hipStream_t stream) {
    const int64_t tiles = (a.n + kCTile - 1) / kCTile;
    if (tiles == 0) {
        compact_empty_kernel<<<(a.num_segments + 256) / 256, 256, 0, stream>>>(a.surv_ptr, a.num_segments);
        return hipGetLastError();
    }
    if (compact_per_snapshot(a.max_snapshot)) {      // every snapshot fits one workgroup
        const int64_t K = a.num_segments / a.stages;
        uint32_t* kept = static_cast<uint32_t*>(a.workspace);
        uint32_t* snap_off = kept + ((K * 4 + 255) & ~(int64_t)255) / 4;
        if (a.staged) {                              // counted and staged by the estimate kernels: only the move is left
            snapshot_offsets_kernel<<<1, 1024, 0, stream>>>(a.kept, K, snap_off);
            move_staged_kernel<<<(unsigned)K, kWave, 0, stream>>>(a, snap_off);
            return hipGetLastError();
        }
        // the smaller workgroup that covers the promised snapshot bound; up to 16 * THREADS snapshots every
        // workgroup adds up the counts before it itself, beyond that one workgroup scans them first
        auto run = [&](auto threads_tag, auto count_tag) {
            constexpr int THREADS = decltype(threads_tag)::value, COUNT = decltype(count_tag)::value;
            const bool scan = K > 16 * THREADS;
            snapshot_kept_kernel<COUNT><<<(unsigned)K, COUNT, 0, stream>>>(a.seg_ptr, a.stages, a.n, (int64_t)THREADS * 16, a.drop, kept, a.status);
            if (scan) snapshot_offsets_kernel<<<1, 1024, 0, stream>>>(kept, K, snap_off);
            compact_local_kernel<THREADS><<<(unsigned)K, THREADS, 0, stream>>>(a, kept, scan ? snap_off : nullptr);
        };
        if (a.max_snapshot <= 4096) run(std::integral_constant<int, 256>{}, std::integral_constant<int, 128>{});
        else run(std::integral_constant<int, 512>{}, std::integral_constant<int, 128>{});
        return hipGetLastError();
    }
    // the stream of tiles: count, (scan), write; no workgroup waits for another
    uint32_t* tile_count = static_cast<uint32_t*>(a.workspace);
    const int64_t row = ((tiles + 1) * 4 + 255) / 256 * 64;          // words per array, 256-byte multiple
    uint32_t* tile_off = tile_count + row;
    TileInfo* info = reinterpret_cast<TileInfo*>(tile_off + row);
    char* after_info = reinterpret_cast<char*>(info) + (((tiles + 1) * (int64_t)sizeof(TileInfo) + 255) & ~(int64_t)255);
    uint32_t* bits = reinterpret_cast<uint32_t*>(after_info);
    uint8_t* slot_keep = reinterpret_cast<uint8_t*>(after_info + (((a.n + 31) / 32 * 4 + 255) & ~(int64_t)255));
    // snapshots promised larger than a tile can stage: the lookups by request id read packed bits
    uint32_t* keep_bits = a.max_snapshot > kStageBytes ? bits : nullptr;
    if (keep_bits) {
        int pb = (int)(((a.n + 31) / 32 + 255) / 256);
        if (pb > 2048) pb = 2048;
        compact_pack_kernel<<<pb, 256, 0, stream>>>(a.drop, a.n, keep_bits);
    }
    compact_count_kernel<<<(unsigned)tiles, kCThreads, 0, stream>>>(a, info, tile_count, slot_keep, keep_bits, tiles);
    const bool scan = tiles > kSelfSumTiles;
    if (scan) compact_tile_scan_kernel<<<1, 1024, 0, stream>>>(tile_count, tiles, tile_off);
    compact_write_kernel<<<(unsigned)tiles, kCThreads, 0, stream>>>(a, info, tile_count, scan ? tile_off : nullptr, slot_keep);
    return hipGetLastError();
}

}  // namespace pard
