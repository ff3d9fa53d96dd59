// Drop-mask stream compaction: the survivor queues (paper Section 4.1: the Request Broker
// keeps or drops each request; the kept ones, in queue order, form the next batches).
//
// keep[j] = !drop[order[j]] for every queue slot j; surv_idx is order filtered by keep;
// surv_ptr[g] = number of kept slots before queue g starts.  Three kernels: per-tile
// kept counts, exclusive scan of the tile counts, per-tile scatter plus the queue
// offsets that fall inside the tile.
#include "pard_device.hpp"

namespace pard {

namespace {

constexpr int kCThreads = 256;
constexpr int kCItems = 16;
constexpr int kCTile = kCThreads * kCItems;

__global__ __launch_bounds__(kCThreads) void compact_count_kernel(CompactArgs A, uint32_t* tile_cnt) {
    __shared__ uint32_t wave_cnt[kCThreads / kWave];
    const int tid = threadIdx.x;
    const int64_t base = (int64_t)blockIdx.x * kCTile;
    uint32_t c = 0;
#pragma unroll
    for (int i = 0; i < kCItems; ++i) {
        const int64_t j = base + i * kCThreads + tid;
        if (j < A.n) {
            const uint32_t r = (uint32_t)A.order[j];
            c += ((int64_t)r < A.n && A.drop[r] == 0) ? 1u : 0u;
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) c += __shfl_xor(c, off);
    if ((tid & 63) == 0) wave_cnt[tid >> 6] = c;
    __syncthreads();
    if (tid == 0) tile_cnt[blockIdx.x] = wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3];
}

// in-place exclusive scan of tile_cnt[0..tiles), total into tile_cnt[tiles]; one workgroup
__global__ __launch_bounds__(1024) void compact_scan_kernel(uint32_t* tile_cnt, int64_t tiles) {
    __shared__ uint32_t wave_tot[16];
    __shared__ uint32_t carry;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) carry = 0;
    __syncthreads();
    for (int64_t base = 0; base < tiles + 1; base += 1024) {
        const int64_t g = base + tid;
        const uint32_t v = g < tiles ? tile_cnt[g] : 0u;
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
        if (g <= tiles) tile_cnt[g] = pre + inc - v;
        __syncthreads();
        if (tid == 1023) carry = pre + inc;
        __syncthreads();
    }
}

__device__ __forceinline__ int64_t lower_bound_i32(const int32_t* a, int64_t count, int64_t value) {
    int64_t lo = 0, hi = count;                 // first index with a[i] >= value
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if ((int64_t)a[mid] < value) lo = mid + 1; else hi = mid;
    }
    return lo;
}

__global__ __launch_bounds__(kCThreads) void compact_scatter_kernel(CompactArgs A, const uint32_t* tile_off,
                                                                    int64_t tiles) {
    __shared__ uint16_t excl_l[kCTile + 2];     // kept slots before each slot of the tile
    __shared__ uint32_t wave_tot[kCThreads / kWave];
    __shared__ int64_t g_range[2];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t tile = blockIdx.x;
    const int64_t base = tile * kCTile;
    const bool last = tile + 1 >= tiles;
    const int64_t left = A.n - base;
    const int valid = (int)(left < 0 ? 0 : (left < kCTile ? left : kCTile));
    const uint32_t off0 = tiles > 0 ? tile_off[tile] : 0u;

    // blocked: thread t owns slots [t*16, t*16+16) of the tile
    int32_t ids[kCItems];
    uint32_t keep_bits = 0, cnt = 0;
#pragma unroll
    for (int i = 0; i < kCItems; ++i) {
        const int e = tid * kCItems + i;
        ids[i] = 0;
        if (e < valid) {
            ids[i] = A.order[base + e];
            const uint32_t r = (uint32_t)ids[i];
            if ((int64_t)r < A.n && A.drop[r] == 0) { keep_bits |= 1u << i; ++cnt; }
        }
    }
    uint32_t inc = cnt;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        uint32_t t = __shfl_up(inc, off);
        if (lane >= off) inc += t;
    }
    if (lane == 63) wave_tot[wave] = inc;
    if (tid == 0) {
        g_range[0] = lower_bound_i32(A.seg_ptr, (int64_t)A.num_segments + 1, base);
        g_range[1] = last ? (int64_t)A.num_segments + 1
                          : lower_bound_i32(A.seg_ptr, (int64_t)A.num_segments + 1, base + kCTile);
    }
    __syncthreads();
    uint32_t run = inc - cnt;
    for (int w = 0; w < wave; ++w) run += wave_tot[w];
#pragma unroll
    for (int i = 0; i < kCItems; ++i) {
        const int e = tid * kCItems + i;
        if (e < valid) {
            excl_l[e] = (uint16_t)run;
            if (keep_bits & (1u << i)) { A.surv_idx[(int64_t)off0 + run] = ids[i]; ++run; }
        }
    }
    // the owner of the last valid slot also records the tile total one past it
    if (valid > 0 && tid == (valid - 1) / kCItems) excl_l[valid] = (uint16_t)run;
    if (valid == 0 && tid == 0) excl_l[0] = 0;
    __syncthreads();
    for (int64_t g = g_range[0] + tid; g < g_range[1]; g += kCThreads) {
        int64_t p = (int64_t)A.seg_ptr[g] - base;
        if (p < 0) p = 0;
        if (p > valid) p = valid;
        A.surv_ptr[g] = (int32_t)(off0 + excl_l[p]);
    }
}

}  // namespace

int64_t compact_workspace_bytes(int64_t n) {
    const int64_t tiles = (n + kCTile - 1) / kCTile;
    return ((tiles + 1) * 4 + 255) & ~(int64_t)255;
}

hipError_t launch_compact(const CompactArgs& a, hipStream_t stream) {
    const int64_t tiles = (a.n + kCTile - 1) / kCTile;
    uint32_t* tile_cnt = static_cast<uint32_t*>(a.workspace);
    if (tiles > 0) {
        compact_count_kernel<<<(unsigned)tiles, kCThreads, 0, stream>>>(a, tile_cnt);
        compact_scan_kernel<<<1, 1024, 0, stream>>>(tile_cnt, tiles);
    }
    compact_scatter_kernel<<<(unsigned)(tiles > 0 ? tiles : 1), kCThreads, 0, stream>>>(a, tile_cnt, tiles);
    return hipGetLastError();
}

}  // namespace pard
