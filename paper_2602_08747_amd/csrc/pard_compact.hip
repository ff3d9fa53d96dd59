// Drop-mask stream compaction: the survivor queues (paper Section 4.1: the Request Broker
// keeps or drops each request; the kept ones, in queue order, form the next batches).
//
// keep[j] = !drop[order[j]] for every queue slot j; surv_idx is order filtered by keep;
// surv_ptr[g] = number of kept slots before queue g starts.
//
// One pass over the data.  A workgroup counts the kept slots of a tile of 4096 queue slots,
// publishes the count, and receives the number of kept slots in all earlier tiles from a
// scan service: one wave of a helper workgroup walks the tile counts in order (64 tiles per
// load, four loads in flight, running total in a register) and hands each tile its offset
// as soon as the tiles up to it have published.  A waiting tile polls one word.  (A
// look-back in which every waiting tile re-reads a window of predecessor words floods the
// memory fabric with polling traffic when ~1500 tiles are resident.)
//
// Tile order: a tile must only wait for tiles that already run.  Workgroups are persistent
// and claim tiles from one of 16 interleaved pools (pool y owns tiles y, y+16, y+32, ... and
// hands them out in increasing order through its own counter; a workgroup uses pool
// blockIdx % 16).  The lowest tile without an offset is then either running or next in line
// in a pool whose workgroups have nothing unfinished left, and publishing a count never
// waits, so every wait ends as long as 17 workgroups of the grid fit on the device.  A single
// ticket counter would give the same order, but atomics on one address cost ~11 ns each here
// (~95 us for 8192 tiles); 16 counters on separate cache lines run in parallel.  The first
// workgroup of pool 0 to arrive becomes the helper.
#include "pard_device.hpp"

namespace pard {

namespace {

constexpr int kCThreads = 256;
constexpr int kCItems = 16;
constexpr int kCTile = kCThreads * kCItems;
constexpr int kCWaves = kCThreads / kWave;
constexpr uint32_t kFlagReady = 1u << 31;              // word has been published
constexpr uint32_t kValueMask = (1u << 30) - 1;
constexpr uint32_t kSpinLimit = 1u << 22;
constexpr int kPools = 16;                             // tile pools (see above)
constexpr int kLook = 4;                               // groups of 64 tile counts the scan service requests per step
constexpr int kPoolStride = 64;                        // counters 256 bytes apart

__global__ void compact_zero_kernel(uint32_t* p, int64_t count) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < count; i += stride) p[i] = 0;
}

// First index in [0, count) with a[i] >= value (count when there is none), found by one
// whole wave: every step probes 64 evenly spaced entries, so 24k entries take 3 dependent
// loads instead of 15.  All 64 lanes must call it together; all return the same result.
__device__ __forceinline__ int64_t wave_lower_bound_i32(const int32_t* a, int64_t count, int64_t value, int lane) {
    int64_t lo = 0, hi = count;
    while (hi > lo) {
        const int64_t chunk = (hi - lo + 63) >> 6;
        int64_t idx = lo + (int64_t)(lane + 1) * chunk - 1;      // last entry of this lane's chunk
        const bool in_range = idx - chunk + 1 < hi;              // the chunk is not empty
        if (idx >= hi) idx = hi - 1;
        const bool ge = in_range && (int64_t)a[idx] >= value;
        const unsigned long long m = __ballot(ge);
        if (m == 0ull) return hi;                                // every entry is smaller
        const int f = __ffsll((long long)m) - 1;                 // first chunk whose last entry is >= value
        const int64_t new_lo = lo + (int64_t)f * chunk;
        int64_t new_hi = new_lo + chunk - 1;                     // that last entry is a valid answer
        if (new_hi > hi - 1) new_hi = hi - 1;
        if (chunk == 1) return new_lo;
        lo = new_lo;
        hi = new_hi;
        // invariant: a[hi] >= value, answer in [lo, hi]; an empty [lo, hi) means the answer is hi
        if (hi == lo) return lo;
    }
    return lo;
}

// The scan service (one wave).  state[t] = ready | kept slots of tile t, written by the tile;
// prefix[t] = ready | kept slots of tiles 0..t-1, written here.
__device__ __forceinline__ void compact_scan_service(const uint32_t* state, uint32_t* prefix, int64_t tiles,
                                                     int lane, uint32_t* status_word) {
    int64_t base = 0;
    uint32_t running = 0, idle = 0;
    while (base < tiles) {
        uint32_t v[kLook];
#pragma unroll
        for (int c = 0; c < kLook; ++c) {
            const int64_t t = base + 64 * c + lane;
            const uint32_t x = __hip_atomic_load(state + (t < tiles ? t : tiles - 1), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            v[c] = t < tiles ? x : kFlagReady;                   // past the end: nothing to add
        }
        int processed = 0;
        bool go = true;
#pragma unroll
        for (int c = 0; c < kLook; ++c) {
            if (!go) continue;
            const unsigned long long ready = __ballot((v[c] & kFlagReady) != 0);
            const int nready = ready == ~0ull ? 64 : __ffsll((long long)~ready) - 1;   // leading published tiles
            const uint32_t val = lane < nready ? (v[c] & kValueMask) : 0u;
            uint32_t inc = val;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const uint32_t t = __shfl_up(inc, off);
                if (lane >= off) inc += t;
            }
            const int64_t t = base + 64 * c + lane;
            if (lane < nready && t < tiles)
                __hip_atomic_store(prefix + t, kFlagReady | ((running + inc - val) & kValueMask), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            running += __shfl(inc, 63);
            processed += nready;
            if (nready < 64) go = false;
        }
        base += processed;
        if (processed == 0) {
            if (++idle > kSpinLimit) { if (lane == 0) atomicOr(status_word, kStatusLookbackTimeout); return; }
            __builtin_amdgcn_s_sleep(2);
        } else {
            idle = 0;
        }
    }
}

// tile_state[0..tiles), tile_prefix[0..tiles): see the scan service; pool_ctr[y * kPoolStride]: next tile of
// pool y; pool_ctr[kPools * kPoolStride]: arrival counter that elects the helper.  All zero at launch.
__global__ __launch_bounds__(kCThreads) void compact_kernel(CompactArgs A, uint32_t* tile_state, uint32_t* tile_prefix,
                                                            uint32_t* pool_ctr, int64_t tiles, int pools,
                                                            uint32_t* status_word) {
    __shared__ __align__(16) uint16_t excl_l[kCTile + 8];   // kept slots of this tile before each slot
    __shared__ uint32_t wave_tot[kCWaves];
    __shared__ uint32_t s_excl;
    __shared__ int64_t s_tile;
    __shared__ int64_t g_range[2];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int pool = (int)(blockIdx.x % (unsigned)pools);
    if (tiles > 0 && pool == 0) {       // the first workgroup of pool 0 to arrive runs the scan service
        if (tid == 0) s_excl = atomicAdd(&pool_ctr[kPools * kPoolStride], 1u);
        __syncthreads();
        const bool helper = s_excl == 0;
        __syncthreads();
        if (helper) {
            if (wave == 0) compact_scan_service(tile_state, tile_prefix, tiles, lane, status_word);
            return;
        }
    }

    while (true) {
    if (tid == 0)
        s_tile = tiles > 0 ? (int64_t)atomicAdd(&pool_ctr[pool * kPoolStride], 1u) * pools + pool
                           : (int64_t)blockIdx.x;          // no requests: one pass for the offsets
    __syncthreads();
    const int64_t tile = s_tile;
    if (tile >= (tiles > 0 ? tiles : 1)) break;
    const int64_t base = tile * kCTile;
    const bool last = tile + 1 >= tiles;
    const int64_t left = A.n - base;
    const int valid = (int)(left < 0 ? 0 : (left < kCTile ? left : kCTile));
    const bool vec = ((reinterpret_cast<uintptr_t>(A.order) | reinterpret_cast<uintptr_t>(A.surv_idx)) & 15) == 0;

    // wave w owns slots [w*1024, (w+1)*1024) of the tile; load k covers 256 of them, 4 per lane
    int32_t ids[4][4];
    uint32_t keep[4], cnt[4];
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
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int e = wave * 1024 + k * 256 + lane * 4;
        keep[k] = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint32_t r = (uint32_t)ids[k][c];
            if (e + c < valid && (int64_t)r < A.n && A.drop[r] == 0) keep[k] |= 1u << c;
        }
        cnt[k] = (uint32_t)__popc(keep[k]);
    }
    // kept slots before this lane's group of 4, inside the wave's 1024 slots
    uint32_t before[4];
    uint32_t carry = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        uint32_t inc = cnt[k];
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t t = __shfl_up(inc, off);
            if (lane >= off) inc += t;
        }
        before[k] = carry + inc - cnt[k];
        carry += __shfl(inc, 63);
    }
    if (lane == 0) wave_tot[wave] = carry;
    if (wave == kCWaves - 1) {          // queues whose offset falls into this tile
        const int64_t g0 = wave_lower_bound_i32(A.seg_ptr, (int64_t)A.num_segments + 1, base, lane);
        if (lane == 0) g_range[0] = g0;
    } else if (wave == kCWaves - 2) {
        const int64_t g1 = last ? (int64_t)A.num_segments + 1
                                : wave_lower_bound_i32(A.seg_ptr, (int64_t)A.num_segments + 1, base + kCTile, lane);
        if (lane == 0) g_range[1] = g1;
    }
    __syncthreads();
    uint32_t wave_before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kCWaves; ++w) {
        const uint32_t t = wave_tot[w];
        if (w < wave) wave_before += t;
        total += t;
    }

    // kept slots in all earlier tiles: publish this tile's count, poll its offset later
    if (tid == 0 && tiles > 0)
        __hip_atomic_store(&tile_state[tile], kFlagReady | total, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // meanwhile: per-slot counts for the queue offsets
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int e = wave * 1024 + k * 256 + lane * 4;
        const uint32_t b0 = wave_before + before[k];
        const uint32_t b1 = b0 + (keep[k] & 1u), b2 = b1 + ((keep[k] >> 1) & 1u), b3 = b2 + ((keep[k] >> 2) & 1u);
        *reinterpret_cast<uint2*>(excl_l + e) = make_uint2(b0 | (b1 << 16), b2 | (b3 << 16));
    }
    if (tid == 0) {
        excl_l[kCTile] = (uint16_t)total;
        uint32_t pv = kFlagReady;
        if (tiles > 0) {
            uint32_t spins = 0;
            while (!((pv = __hip_atomic_load(&tile_prefix[tile], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) & kFlagReady)) {
                if (++spins > kSpinLimit) { atomicOr(status_word, kStatusLookbackTimeout); break; }
                __builtin_amdgcn_s_sleep(2);
            }
        }
        s_excl = pv & kValueMask;
    }
    __syncthreads();
    const uint32_t off0 = s_excl;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        uint32_t o = off0 + wave_before + before[k];
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (keep[k] & (1u << c)) { A.surv_idx[o] = ids[k][c]; ++o; }
    }
    // queue offsets that fall into this tile (the last tile also takes those equal to n)
    for (int64_t g = g_range[0] + tid; g < g_range[1]; g += kCThreads) {
        int64_t p = (int64_t)A.seg_ptr[g] - base;
        if (p < 0) p = 0;
        if (p > valid) p = valid;
        A.surv_ptr[g] = (int32_t)(off0 + (p >= valid ? total : (uint32_t)excl_l[p]));
    }
    __syncthreads();                    // LDS is reused by the next tile
    if (tiles == 0) break;
    }
}

}  // namespace

int64_t compact_workspace_bytes(int64_t n) {
    const int64_t tiles = (n + kCTile - 1) / kCTile;
    return (int64_t)(kPools + 1) * kPoolStride * 4 + 2 * (((tiles + 1) * 4 + 255) & ~(int64_t)255);
}

int compact_blocks_per_cu() {
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, compact_kernel, kCThreads, 0) != hipSuccess || per_cu < 1) {
        (void)hipGetLastError();
        per_cu = 1;
    }
    return per_cu;
}

hipError_t launch_compact(const CompactArgs& a, hipStream_t stream) {
    const int64_t tiles = (a.n + kCTile - 1) / kCTile;
    uint32_t* pool_ctr = static_cast<uint32_t*>(a.workspace);
    const int64_t row = ((tiles + 1) * 4 + 255) / 256 * 64;          // words per array, 256-byte multiple
    uint32_t* tile_state = pool_ctr + (kPools + 1) * kPoolStride;
    uint32_t* tile_prefix = tile_state + row;
    const int64_t words = (int64_t)(kPools + 1) * kPoolStride + 2 * row;
    int zb = (int)((words + 255) / 256);
    if (zb > 1024) zb = 1024;
    compact_zero_kernel<<<zb, 256, 0, stream>>>(pool_ctr, words);
    int64_t grid = a.resident_blocks > 0 ? a.resident_blocks : 1;     // persistent: what the device holds at once
    if (grid > tiles) grid = tiles;
    if (grid < 1) grid = 1;
    const int pools = grid < kPools ? (int)grid : kPools;                 // pool 0 then holds at least two workgroups
    if (tiles > 0) grid += 1;                                             // one workgroup becomes the scan service
    compact_kernel<<<(unsigned)grid, kCThreads, 0, stream>>>(a, tile_state, tile_prefix, pool_ctr, tiles, pools, a.status);
    return hipGetLastError();
}

}  // namespace pard
