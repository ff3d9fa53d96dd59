// Drop-mask stream compaction: the survivor queues (paper Section 4.1: the Request Broker
// keeps or drops each request; the kept ones, in queue order, form the next batches).
//
// keep[j] = !drop[order[j]] for every queue slot j; surv_idx is order filtered by keep;
// surv_ptr[g] = number of kept slots before queue g starts.
//
// One pass over the data: a workgroup counts the kept slots of a tile of 4096 queue slots,
// publishes the count, and obtains the number of kept slots in all earlier tiles by a
// decoupled look-back (one wave inspects 64 predecessor tiles at a time).
//
// Tile order: a tile may only wait for tiles that already run.  Workgroups are persistent
// and claim tiles from one of 16 interleaved pools (pool y owns tiles y, y+16, y+32, ... and
// hands them out in increasing order through its own counter; a workgroup uses pool
// blockIdx % 16).  The lowest unfinished tile is then either running or next in line in a
// pool whose workgroups have nothing unfinished left, so every wait ends as long as 16
// workgroups of the grid fit on the device.  A single ticket counter would give the same
// order, but atomics on one address cost ~11 ns each here (~95 us for 8192 tiles, more
// than the rest of the kernel); 16 counters on separate cache lines run in parallel.
#include "pard_device.hpp"

namespace pard {

namespace {

constexpr int kCThreads = 256;
constexpr int kCItems = 16;
constexpr int kCTile = kCThreads * kCItems;
constexpr int kCWaves = kCThreads / kWave;
constexpr uint32_t kFlagAggregate = 1u << 30;          // tile published its own count
constexpr uint32_t kFlagInclusive = 2u << 30;          // tile published the running total
constexpr uint32_t kValueMask = (1u << 30) - 1;
constexpr uint32_t kSpinLimit = 1u << 22;
constexpr int kPools = 16;                             // tile pools (see above)
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

__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

// tile_state[0..tiles): look-back words; pool_ctr[y * kPoolStride]: next tile of pool y.  All zero at launch.
__global__ __launch_bounds__(kCThreads) void compact_kernel(CompactArgs A, uint32_t* tile_state, uint32_t* pool_ctr,
                                                            int64_t tiles, int pools, uint32_t* status_word) {
    __shared__ __align__(16) uint16_t excl_l[kCTile + 8];   // kept slots of this tile before each slot
    __shared__ uint32_t wave_tot[kCWaves];
    __shared__ uint32_t s_excl;
    __shared__ int64_t s_tile;
    __shared__ int64_t g_range[2];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int pool = (int)(blockIdx.x % (unsigned)pools);

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

    // kept slots in all earlier tiles
    if (wave == 0) {
        uint32_t excl = 0;
        if (tiles > 0) {
            if (tile == 0) {
                if (lane == 0) __hip_atomic_store(&tile_state[0], kFlagInclusive | total, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else {
                if (lane == 0) __hip_atomic_store(&tile_state[tile], kFlagAggregate | total, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                int64_t window = tile - 1;                  // lane l inspects tile window - l
                bool done = false;
                uint32_t spins = 0;
                while (!done) {
                    const int64_t t = window - lane;
                    uint32_t v = kFlagInclusive;            // tiles before the first count as a finished zero
                    if (t >= 0) v = __hip_atomic_load(&tile_state[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (__ballot((v & ~kValueMask) == 0) != 0ull) {     // someone has not published yet
                        if (++spins > kSpinLimit) {
                            if (lane == 0) atomicOr(status_word, kStatusLookbackTimeout);
                            break;
                        }
                        __builtin_amdgcn_s_sleep(1);
                        continue;
                    }
                    const unsigned long long inc_mask = __ballot((v & ~kValueMask) == kFlagInclusive);
                    if (inc_mask != 0ull) {
                        const int first = __ffsll((long long)inc_mask) - 1;   // nearest tile with a running total
                        excl += wave_sum(lane <= first ? (v & kValueMask) : 0u);
                        done = true;
                    } else {
                        excl += wave_sum(v & kValueMask);
                        window -= 64;
                    }
                }
                if (lane == 0) __hip_atomic_store(&tile_state[tile], kFlagInclusive | ((excl + total) & kValueMask),
                                                  __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        if (lane == 0) s_excl = excl;
    }
    // meanwhile: per-slot counts for the queue offsets
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int e = wave * 1024 + k * 256 + lane * 4;
        const uint32_t b0 = wave_before + before[k];
        const uint32_t b1 = b0 + (keep[k] & 1u), b2 = b1 + ((keep[k] >> 1) & 1u), b3 = b2 + ((keep[k] >> 2) & 1u);
        *reinterpret_cast<uint2*>(excl_l + e) = make_uint2(b0 | (b1 << 16), b2 | (b3 << 16));
    }
    if (tid == 0) excl_l[kCTile] = (uint16_t)total;
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
    return (int64_t)kPools * kPoolStride * 4 + (((tiles + 1) * 4 + 255) & ~(int64_t)255);
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
    uint32_t* tile_state = pool_ctr + kPools * kPoolStride;
    const int64_t words = (int64_t)kPools * kPoolStride + tiles + 1;
    int zb = (int)((words + 255) / 256);
    if (zb > 1024) zb = 1024;
    compact_zero_kernel<<<zb, 256, 0, stream>>>(pool_ctr, words);
    int64_t grid = a.resident_blocks > 0 ? a.resident_blocks : 1;     // persistent: what the device holds at once
    if (grid > tiles) grid = tiles;
    if (grid < 1) grid = 1;
    const int pools = grid < kPools ? (int)grid : kPools;
    compact_kernel<<<(unsigned)grid, kCThreads, 0, stream>>>(a, tile_state, pool_ctr, tiles, pools, a.status);
    return hipGetLastError();
}

}  // namespace pard
