// Host-side plan building: validation of the pipeline description, DAG -> path
// expansion, per-stage constants.  Pure C++17, no HIP, so that the same code can be
// compiled into a CPU-only test shim.
//
// Paper basis: a pipeline is a set of modules with predecessor/successor lists
// (Section 4, "Implementation"); for a DAG the latency is estimated along each
// subsequent path and the maximum is taken (Section 3.2, paragraph before Eq.(4)).
#pragma once

#include <cstddef>
#include <cstdint>
#include <vector>

#include "../../include/pard.h"

namespace pard {

// Per-(DAG, stage) constants as the kernels read them (48 bytes).
struct StageRec {
    int32_t B;        // batch size, 1..64
    int32_t W;        // workers, 1..2^20
    int32_t latB;     // lat[B]: latency of a full batch
    int32_t mode;     // PARD_ORDER_* in bits 0..7, kStageFast in bit 8
    uint32_t mB;      // multiplier for floor(x / B), x < 2^32
    uint32_t shB;     // shift pair for it: sh1 | sh2 << 8
    uint32_t mW;      // multiplier for floor(x / W), x < 2^32
    uint32_t shW;
    float rcpB;       // 1/B and 1/W rounded to nearest, for the short-queue fast path
    float rcpW;
    uint32_t aW;      // latB / W
    uint32_t bW;      // latB % W
};

// Set when W <= 256 and latB / W < 2^18: for queue positions below 2^13 the wait term
// floor(ceil(a/B) * latB / W) can then be formed exactly from 24-bit multiplies and two
// float reciprocal multiplies (see stage_cost_short in pard_device.hpp).
constexpr int32_t kStageFast = 1 << 8;

// Division of a 32-bit unsigned integer by an invariant divisor d >= 1 via one
// high multiply (Granlund & Montgomery, "Division by invariant integers using
// multiplication", Fig. 4.1, N = 32):
//   l = ceil(log2 d), m = floor(2^32 (2^l - d) / d) + 1, sh1 = min(l,1), sh2 = max(l-1,0)
//   t = mulhi(m, n);  q = (t + ((n - t) >> sh1)) >> sh2
struct Magic32 {
    uint32_t m;
    uint32_t sh;      // sh1 | sh2 << 8
};

inline Magic32 magic_u32(uint32_t d) {
    uint32_t l = 0;
    while (l < 32 && ((uint64_t)1 << l) < d) ++l;
    uint64_t num = (((uint64_t)1 << l) - d) << 32;
    uint32_t m = (uint32_t)(num / d) + 1u;
    uint32_t sh1 = l < 1 ? l : 1;
    uint32_t sh2 = l > 1 ? l - 1 : 0;
    return Magic32{m, sh1 | (sh2 << 8)};
}

inline uint32_t magic_div(uint32_t n, Magic32 k) {
    uint32_t t = (uint32_t)(((uint64_t)k.m * n) >> 32);
    return (t + ((n - t) >> (k.sh & 0xFF))) >> (k.sh >> 8);
}

struct HostPlan {
    int32_t K = 0, S = 0, shared = 1, D = 0;
    bool any_fcfs = false;
    int32_t uniform_mode = -1;              // >= 0 when every stage uses that mode
    int64_t total_paths = 0;
    int32_t max_path_len = 0;
    int32_t max_entries_per_dag = 0;
    std::vector<StageRec> recs;             // [D*S]
    std::vector<int32_t> lat;               // [D*S*64]
    std::vector<int32_t> dag_path_ptr;      // [D+1]   first path of each DAG
    std::vector<int32_t> path_ptr;          // [P+1]   path CSR: offsets into entry_stage
    std::vector<int32_t> dag_entry_ptr;     // [D+1]   first path entry of each DAG
    std::vector<int32_t> entry_stage;       // [E]     stage ids along the paths
    std::vector<int32_t> entry_end;         // [E]     one past the last entry of the entry's path
    std::vector<int32_t> entry_dag;         // [E]     the DAG an entry belongs to
    int32_t max_lat = 0;                    // largest latency-table entry
    // Per-module SLO split (Section 5.1, Clipper++): summed execution durations lat[B] along the longest way from a
    // source to a stage (the stage included) and along the longest whole path through it.
    std::vector<int64_t> split_in, split_whole;   // [D*S]
    bool split_fits = true;                 // every such sum is below 2^30 (products with 33-bit times fit 64 bits)
    bool short_form_everywhere = true;      // every stage is kStageFast with latB / W < 2^17: wait + execution of a
                                            // short queue fit 32 bits without a carry
};

// Validates one DAG and appends its source-to-sink paths.  Returns a pard_status.
inline int expand_dag(int32_t S, const int32_t* rp, const int32_t* col, HostPlan& hp) {
    if (rp[0] != 0) return PARD_E_BAD_DAG;
    for (int s = 0; s < S; ++s)
        if (rp[s + 1] < rp[s]) return PARD_E_BAD_DAG;
    if (rp[S] > 0 && col == nullptr) return PARD_E_NULL;
    std::vector<int32_t> indeg(S, 0);
    for (int s = 0; s < S; ++s)
        for (int32_t e = rp[s]; e < rp[s + 1]; ++e) {
            int32_t t = col[e];
            if (t < 0 || t >= S || t == s) return PARD_E_BAD_DAG;
            indeg[t] += 1;
        }
    // acyclic?  peel sources (Kahn)
    {
        std::vector<int32_t> left(indeg), ready;
        for (int s = 0; s < S; ++s) if (!left[s]) ready.push_back(s);
        int peeled = 0;
        while (!ready.empty()) {
            int32_t v = ready.back();
            ready.pop_back();
            ++peeled;
            for (int32_t e = rp[v]; e < rp[v + 1]; ++e)
                if (--left[col[e]] == 0) ready.push_back(col[e]);
        }
        if (peeled != S) return PARD_E_BAD_DAG;
    }
    // iterative depth-first walk from every source; emit a path at every sink
    int32_t paths_here = 0, entries_here = 0;
    std::vector<int32_t> node(S + 1), edge(S + 1);
    for (int src = 0; src < S; ++src) {
        if (indeg[src]) continue;
        int depth = 0;
        node[0] = src;
        edge[0] = rp[src];
        while (depth >= 0) {
            int32_t v = node[depth];
            if (rp[v] == rp[v + 1]) {                       // sink: the stack is a complete path
                int32_t len = depth + 1;
                if (paths_here + 1 > PARD_MAX_PATHS_PER_DAG ||
                    entries_here + len > PARD_MAX_PATH_ENTRIES_PER_DAG)
                    return PARD_E_TOO_MANY_PATHS;
                int32_t first = (int32_t)hp.entry_stage.size();
                for (int i = 0; i < len; ++i) {
                    hp.entry_stage.push_back(node[i]);
                    hp.entry_end.push_back(first + len);
                }
                hp.path_ptr.push_back(first + len);
                paths_here += 1;
                entries_here += len;
                if (len > hp.max_path_len) hp.max_path_len = len;
                --depth;
                continue;
            }
            if (edge[depth] == rp[v + 1]) { --depth; continue; }
            int32_t t = col[edge[depth]++];
            ++depth;
            node[depth] = t;
            edge[depth] = rp[t];
        }
    }
    hp.total_paths += paths_here;
    if (entries_here > hp.max_entries_per_dag) hp.max_entries_per_dag = entries_here;
    return PARD_OK;
}

inline int build_host_plan(const pard_plan_desc_t* d, HostPlan& hp) {
    if (!d) return PARD_E_NULL;
    if (d->num_snapshots < 1 || d->num_stages < 1 || d->num_stages > PARD_MAX_STAGES)
        return PARD_E_BAD_SHAPE;
    if (!d->dag_row_ptr || !d->batch || !d->workers || !d->lat_us || !d->order_mode) return PARD_E_NULL;
    hp.K = d->num_snapshots;
    hp.S = d->num_stages;
    hp.shared = d->dag_shared ? 1 : 0;
    hp.D = hp.shared ? 1 : hp.K;
    const int32_t S = hp.S;
    const int64_t DS = (int64_t)hp.D * S;
    hp.recs.resize((size_t)DS);
    hp.lat.assign(d->lat_us, d->lat_us + DS * PARD_LAT_ENTRIES);
    int32_t first_mode = d->order_mode[0];
    bool uniform = true;
    for (int64_t i = 0; i < DS; ++i) {
        int32_t B = d->batch[i], W = d->workers[i], M = d->order_mode[i];
        if (B < 1 || B > PARD_LAT_ENTRIES) return PARD_E_BAD_BATCH;
        if (W < 1 || W > PARD_MAX_WORKERS) return PARD_E_BAD_WORKERS;
        if (M != PARD_ORDER_LBF && M != PARD_ORDER_HBF && M != PARD_ORDER_FCFS) return PARD_E_BAD_MODE;
        for (int b = 0; b < PARD_LAT_ENTRIES; ++b)
            if (d->lat_us[i * PARD_LAT_ENTRIES + b] < 0) return PARD_E_BAD_LATENCY;
        if (M == PARD_ORDER_FCFS) hp.any_fcfs = true;
        if (M != first_mode) uniform = false;
        Magic32 kb = magic_u32((uint32_t)B), kw = magic_u32((uint32_t)W);
        const int32_t latB = d->lat_us[i * PARD_LAT_ENTRIES + B - 1];
        const uint32_t aW = (uint32_t)latB / (uint32_t)W, bW = (uint32_t)latB % (uint32_t)W;
        const int32_t fast = (W <= 256 && aW < (1u << 18)) ? kStageFast : 0;
        if (!fast || aW >= (1u << 17)) hp.short_form_everywhere = false;
        hp.recs[(size_t)i] = StageRec{B, W, latB, M | fast, kb.m, kb.sh, kw.m, kw.sh,
                                      1.0f / (float)B, 1.0f / (float)W, aW, bW};
    }
    hp.uniform_mode = uniform ? first_mode : -1;
    for (int32_t v : hp.lat) if (v > hp.max_lat) hp.max_lat = v;
    hp.dag_path_ptr.assign(1, 0);
    hp.dag_entry_ptr.assign(1, 0);
    hp.path_ptr.assign(1, 0);
    int64_t col_base = 0;
    for (int32_t g = 0; g < hp.D; ++g) {
        const int32_t* rp = d->dag_row_ptr + (int64_t)g * (S + 1);
        int rc = expand_dag(S, rp, d->dag_col ? d->dag_col + col_base : nullptr, hp);
        if (rc != PARD_OK) return rc;
        col_base += rp[S];
        {
            // longest way in and out of every stage, over the paths just listed (every stage lies on one)
            std::vector<int64_t> in(S, 0), out(S, 0);
            const size_t e0 = (size_t)hp.dag_entry_ptr.back(), e1 = hp.entry_stage.size();
            for (size_t first = e0; first < e1;) {
                const size_t end = (size_t)hp.entry_end[first];
                int64_t total = 0;
                for (size_t e = first; e < end; ++e) total += hp.recs[(size_t)g * S + hp.entry_stage[e]].latB;
                int64_t run = 0;
                for (size_t e = first; e < end; ++e) {
                    const int32_t v = hp.entry_stage[e];
                    run += hp.recs[(size_t)g * S + v].latB;
                    if (run > in[v]) in[v] = run;
                    if (total - run > out[v]) out[v] = total - run;
                }
                first = end;
            }
            for (int32_t v = 0; v < S; ++v) {
                hp.split_in.push_back(in[v]);
                hp.split_whole.push_back(in[v] + out[v]);
                if (in[v] + out[v] >= ((int64_t)1 << 30)) hp.split_fits = false;
            }
        }
        hp.dag_path_ptr.push_back((int32_t)(hp.path_ptr.size() - 1));
        hp.dag_entry_ptr.push_back((int32_t)hp.entry_stage.size());
        hp.entry_dag.resize(hp.entry_stage.size(), g);
        if (hp.entry_stage.size() > (size_t)0x7fffffff - PARD_MAX_PATH_ENTRIES_PER_DAG) return PARD_E_TOO_MANY_PATHS;
    }
    return PARD_OK;
}

}  // namespace pard
