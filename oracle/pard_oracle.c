/*
 * TEST INFRASTRUCTURE -- plain CPU oracle for the batched latency estimate, drop
 * decision and survivor compaction of PARD's proactive request dropping.
 *
 * This file is the slow, obviously-correct statement of what the GPU library
 * must compute.  It is used only by the tests, the smoke check and the
 * benchmark's CPU-baseline leg; the product path never calls it and shares no
 * code, header, table or helper with it.
 *
 * What it follows (paper sections):
 *   - Section 3.2 Eq.(1): end-to-end latency = preceding + current + subsequent modules.
 *   - Section 3.2 Eq.(2): per-module latency = queueing delay + batch wait + execution.
 *   - Section 3.2 Eq.(4) and the DAG sentence before it: the estimate is the sum of
 *     the per-module terms along a downstream path; for a DAG, the maximum over all
 *     downstream paths.
 *   - Section 3.3: the queue is ordered by remaining latency budget (low budget first
 *     or high budget first); arrival order is the paper's FCFS ablation (Section 5.3).
 *   - Drop when the estimated end-to-end latency exceeds the SLO, i.e. when
 *     now + estimate lies after the request's deadline (Section 3.2, end).
 *
 * Snapshot form (the paper's runtime averages need history, a snapshot has none):
 * the wait of a request with `a` requests ahead of it in a stage with batch size B,
 * W workers and batch-latency table lat[] is  floor(ceil(a/B) * lat[B] / W), and its
 * execution latency is lat[min(B, a+1)].  In its own stage `a` is its queue position;
 * in every downstream stage `a` is that stage's whole queue length.  All arithmetic
 * is integer microseconds in 128-bit integers, so nothing can overflow; results are
 * clamped to INT32_MAX on output only.
 *
 * The State Planner's part (Section 3.2 Eq.(4), "Batch wait estimation"): the latency of
 * the modules after the current one is the sum of their queueing delays and execution
 * durations plus w, the lambda-quantile of the aggregated batch wait time, which the paper
 * obtains by random sampling over the collected arrival process (M = 10,000 by default).
 * pard_oracle_sub_latency() computes that per (snapshot, stage), with the paper's ablation
 * variants (-lower, -upper, -sf, -back; Section 5.1 Table of baselines, Section 5.3); see
 * the comment at the function for the sampling rule.  Its pins: the quantiles the paper
 * prints for a four-module pipeline (0.31, 0.28, 0.22, 0.10 of the summed durations),
 * an independent numpy brute force, closed forms and identities (tests/test_oracle_sub.py).
 *
 * Adaptive priority with delayed transition (Section 3.3): pard_oracle_priority_modes()
 * decides per (snapshot, stage) between High-Budget-First and Low-Budget-First from the
 * module load factor mu = T_in / T_m with the two thresholds 1 +- epsilon; see the comment
 * at the function.  Pins: hand-worked series, closed forms and an independent Python brute
 * force with exact rationals (tests/test_oracle_priority.py); the paper prints no value for it
 * and its algorithm listing is absent, so parity with the paper is unpinned for this function.
 *
 * Ranked downstream positions (pard_oracle_estimate_drop_ranked): the snapshot form above lets a
 * request join the back of every later queue; the paper's queues are kept in budget order
 * (Section 3.3), so this variant counts, in a later queue, only the requests that order would
 * serve before the newcomer.  A reading, not a formula of the paper: parity with the paper is
 * unpinned; pinned by a brute force and by the cases in which it must equal the plain estimate
 * or differ from it by a known amount (tests/test_oracle_ranked.py).
 *
 * Monitored queueing delay (Section 3.2, State Planner, first item and its footnote: a sliding
 * window over the recent queueing delays, 5 s and linearly weighted by default):
 * pard_oracle_queue_delay() gives q_i per (snapshot, stage) from time-stamped delay samples,
 * and pard_oracle_sub_latency() takes those q_i in place of the snapshot stand-in when they
 * are passed.  The paper prints no value for it, so parity with the paper is unpinned; the pins
 * are hand-worked windows, the closed form of a linearly weighted mean over equally spaced
 * samples, and an exact-rational brute force (tests/test_oracle_window.py).
 *
 * Reactive baselines on the same snapshot (Section 5.1 "Baselines"): pard_oracle_nexus_drop() is the
 * reactive policy the paper describes for Nexus (scan the queue in arrival order with a window of one
 * batch, stop at the first window whose requests can all still finish the current module, drop everything
 * before it); pard_oracle_clipper_drop() is Clipper++ (the end-to-end SLO divided among the modules in
 * proportion to their execution durations, a request is dropped once it has used up the budget of the
 * modules up to and including its own).  The paper prints no value for either, and a snapshot has to read
 * both rules (see the comments at the functions): parity with the paper is unpinned; the pins are
 * hand-worked queues, closed forms and independent Python brute forces (tests/test_oracle_reactive.py).
 *
 * Parity status: no value in the paper pins the estimate/drop path (it prints none for it).
 * The pins are brute force on tiny inputs, closed forms, invariants and a hand-worked
 * vector (tests/test_oracle_*.py).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define LAT_ENTRIES 64
#define MODE_LBF 0
#define MODE_HBF 1
#define MODE_FCFS 2

typedef __int128 wide_t;

typedef struct {
    int64_t key;
    int32_t idx;
} queued_t;

static int cmp_queued(const void* pa, const void* pb) {
    const queued_t* a = (const queued_t*)pa;
    const queued_t* b = (const queued_t*)pb;
    if (a->key != b->key) return a->key < b->key ? -1 : 1;
    if (a->idx != b->idx) return a->idx < b->idx ? -1 : 1;   /* ties: original index ascending */
    return 0;
}

/* A stage id outside [0,S) is a caller error; both implementations agree to read it
 * as the nearest valid stage so that nothing is ever indexed out of bounds. */
static int clamp_stage(int32_t s, int S) {
    if (s < 0) return 0;
    if (s >= S) return S - 1;
    return s;
}

/* Eq.(2) in snapshot form: wait (queueing + batch wait) plus execution, with `a`
 * requests ahead.  lat points at the stage's 64-entry table, lat[b-1] = latency of a
 * batch of b. */
static wide_t stage_cost(const int32_t* lat, int32_t B, int32_t W, int64_t a) {
    int64_t batches_ahead = (a + B - 1) / B;                    /* ceil(a / B) */
    wide_t wait = ((wide_t)batches_ahead * (wide_t)lat[B - 1]) / (wide_t)W;
    int64_t b_seen = (a + 1 < B) ? a + 1 : B;                   /* batch the request runs in */
    return wait + (wide_t)lat[b_seen - 1];
}

/* ---- all source-to-sink paths of one DAG, by depth-first search -------------- */

typedef struct {
    int32_t* ptr;      /* [P+1] */
    int32_t* stage;    /* [ptr[P]] */
    int64_t P, cap_ptr, len, cap_len;
    int err;
} paths_t;

static void paths_push(paths_t* ps, const int32_t* stack, int depth) {
    if (ps->P + 2 > ps->cap_ptr) {
        ps->cap_ptr = ps->cap_ptr ? ps->cap_ptr * 2 : 16;
        ps->ptr = (int32_t*)realloc(ps->ptr, sizeof(int32_t) * (size_t)ps->cap_ptr);
    }
    if (ps->len + depth > ps->cap_len) {
        while (ps->len + depth > ps->cap_len) ps->cap_len = ps->cap_len ? ps->cap_len * 2 : 64;
        ps->stage = (int32_t*)realloc(ps->stage, sizeof(int32_t) * (size_t)ps->cap_len);
    }
    if (ps->P == 0) ps->ptr[0] = 0;
    memcpy(ps->stage + ps->len, stack, sizeof(int32_t) * (size_t)depth);
    ps->len += depth;
    ps->P += 1;
    ps->ptr[ps->P] = (int32_t)ps->len;
}

static void paths_dfs(paths_t* ps, int S, const int32_t* row_ptr, const int32_t* col,
                      int32_t* stack, int depth) {
    if (ps->err) return;
    if (depth > S) { ps->err = 1; return; }                     /* longer than S stages: a cycle */
    int32_t v = stack[depth - 1];
    if (row_ptr[v] == row_ptr[v + 1]) { paths_push(ps, stack, depth); return; }
    for (int32_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e) {
        int32_t w = col[e];
        if (w < 0 || w >= S) { ps->err = 2; return; }
        stack[depth] = w;
        paths_dfs(ps, S, row_ptr, col, stack, depth + 1);
    }
}

static int enumerate_paths(int S, const int32_t* row_ptr, const int32_t* col, paths_t* ps) {
    memset(ps, 0, sizeof(*ps));
    int32_t* indeg = (int32_t*)calloc((size_t)S, sizeof(int32_t));
    int32_t* stack = (int32_t*)malloc(sizeof(int32_t) * (size_t)(S + 2));
    for (int32_t e = row_ptr[0]; e < row_ptr[S]; ++e)
        if (col[e] >= 0 && col[e] < S) indeg[col[e]] += 1; else ps->err = 2;
    /* acyclic check (Kahn): peel stages whose predecessors are all peeled */
    if (!ps->err) {
        int32_t* left = (int32_t*)malloc(sizeof(int32_t) * (size_t)(S + 1));
        int32_t* ready = (int32_t*)malloc(sizeof(int32_t) * (size_t)(S + 1));
        int nready = 0, peeled = 0;
        for (int s = 0; s < S; ++s) { left[s] = indeg[s]; if (!left[s]) ready[nready++] = s; }
        while (nready) {
            int32_t v = ready[--nready];
            peeled += 1;
            for (int32_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e)
                if (--left[col[e]] == 0) ready[nready++] = col[e];
        }
        if (peeled != S) ps->err = 1;
        free(left);
        free(ready);
    }
    int nsrc = 0;
    for (int s = 0; s < S && !ps->err; ++s) {
        if (indeg[s] != 0) continue;
        nsrc += 1;
        stack[0] = s;
        paths_dfs(ps, S, row_ptr, col, stack, 1);
    }
    if (!ps->err && nsrc == 0 && S > 0) ps->err = 1;            /* no source: every stage is on a cycle */
    free(indeg);
    free(stack);
    return ps->err;
}

static void paths_free(paths_t* ps) {
    free(ps->ptr);
    free(ps->stage);
}

/* Exported for the tests: number of source-to-sink paths, longest path length (in
 * stages) and, when out arrays are given, the paths themselves.  Returns 0, or
 * 1 = cycle, 2 = edge out of range, 3 = output capacity too small. */
int pard_oracle_paths(int32_t S, const int32_t* row_ptr, const int32_t* col,
                      int64_t* num_paths, int64_t* max_len,
                      int32_t* out_ptr, int64_t cap_ptr, int32_t* out_stage, int64_t cap_stage) {
    paths_t ps;
    int err = enumerate_paths(S, row_ptr, col, &ps);
    if (err) { paths_free(&ps); return err; }
    int64_t mx = 0;
    for (int64_t p = 0; p < ps.P; ++p) {
        int64_t L = ps.ptr[p + 1] - ps.ptr[p];
        if (L > mx) mx = L;
    }
    if (num_paths) *num_paths = ps.P;
    if (max_len) *max_len = mx;
    if (out_ptr && out_stage) {
        if (cap_ptr < ps.P + 1 || cap_stage < ps.len) { paths_free(&ps); return 3; }
        if (ps.P) memcpy(out_ptr, ps.ptr, sizeof(int32_t) * (size_t)(ps.P + 1)); else out_ptr[0] = 0;
        if (ps.len) memcpy(out_stage, ps.stage, sizeof(int32_t) * (size_t)ps.len);
    }
    paths_free(&ps);
    return 0;
}

/* Exported for the tests: the per-stage cost alone, clamped to INT64_MAX. */
int64_t pard_oracle_stage_cost(const int32_t* lat, int32_t B, int32_t W, int64_t a) {
    wide_t c = stage_cost(lat, B, W, a);
    wide_t cap = (wide_t)INT64_MAX;
    return (int64_t)(c > cap ? cap : c);
}

/*
 * Estimate + drop decision for K snapshots.
 *
 * Plan arrays (D = dag_shared ? 1 : K copies): row_ptr[D*(S+1)] with offsets relative
 * to each DAG's own col block (blocks are concatenated in order), batch[D*S],
 * workers[D*S], lat[D*S*64], mode[D*S].
 * Snapshot arrays: arrival/deadline/stage[n], snap_ptr[K+1], now[K].
 * Outputs: est[n], drop[n] in request order; order[n] (sorted position -> request id),
 * seg_ptr[K*S+1] offsets of the (snapshot, stage) queues inside order.
 * Returns 0, or a positive code for a malformed DAG.
 */
static int estimate_drop_impl(
        int32_t K, int32_t S, int32_t dag_shared,
        const int32_t* row_ptr, const int32_t* col,
        const int32_t* batch, const int32_t* workers, const int32_t* lat, const int32_t* mode,
        int64_t n, const int32_t* arrival, const int32_t* deadline, const int32_t* stage,
        const int32_t* snap_ptr, const int32_t* now, const int64_t* sub, int consistent, int ranked,
        int32_t* est, uint8_t* drop, int32_t* order, int32_t* seg_ptr,
        int32_t nthreads) {
    (void)n;
    if (nthreads < 1) nthreads = 1;
    int status = 0;
    /* start of each DAG's block inside col */
    int64_t D = dag_shared ? 1 : K;
    int64_t* col_base = (int64_t*)malloc(sizeof(int64_t) * (size_t)(D + 1));
    col_base[0] = 0;
    for (int64_t d = 0; d < D; ++d) col_base[d + 1] = col_base[d] + row_ptr[d * (S + 1) + S];

    for (int32_t u = 0; u < K; ++u) {
        int64_t d = dag_shared ? 0 : u;
        const int32_t* rp = row_ptr + d * (S + 1);
        const int32_t* cl = col + col_base[d];
        const int32_t* B = batch + d * S;
        const int32_t* Wk = workers + d * S;
        const int32_t* L = lat + d * S * LAT_ENTRIES;
        const int32_t* M = mode + d * S;
        int64_t lo = snap_ptr[u], hi = snap_ptr[u + 1];
        int64_t m = hi - lo;

        /* 1. paths */
        paths_t ps;
        int err = enumerate_paths(S, rp, cl, &ps);
        if (err) { status = err; paths_free(&ps); break; }

        /* 2. queues: requests of this snapshot grouped by current stage */
        int64_t* qlen = (int64_t*)calloc((size_t)S, sizeof(int64_t));
        for (int64_t r = lo; r < hi; ++r) qlen[clamp_stage(stage[r], S)] += 1;
        int64_t* qstart = (int64_t*)malloc(sizeof(int64_t) * (size_t)(S + 1));
        qstart[0] = 0;
        for (int s = 0; s < S; ++s) qstart[s + 1] = qstart[s] + qlen[s];
        queued_t* q = (queued_t*)malloc(sizeof(queued_t) * (size_t)(m > 0 ? m : 1));
        int64_t* fill = (int64_t*)calloc((size_t)S, sizeof(int64_t));
        for (int64_t r = lo; r < hi; ++r) {
            int s = clamp_stage(stage[r], S);
            int64_t key;
            if (M[s] == MODE_HBF) key = -(int64_t)deadline[r];       /* largest budget first */
            else if (M[s] == MODE_FCFS) key = (int64_t)arrival[r];   /* arrival order */
            else key = (int64_t)deadline[r];                         /* smallest budget first */
            queued_t* slot = &q[qstart[s] + fill[s]++];
            slot->key = key;
            slot->idx = (int32_t)r;
        }
        /* 3. order every queue by (key, original index) */
        #pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
        for (int s = 0; s < S; ++s)
            qsort(q + qstart[s], (size_t)qlen[s], sizeof(queued_t), cmp_queued);
        for (int s = 0; s < S; ++s) seg_ptr[(int64_t)u * S + s] = (int32_t)(lo + qstart[s]);
        for (int64_t j = 0; j < m; ++j) order[lo + j] = q[j].idx;

        /* 4.-6. per request: maximum over the paths through its stage.
         * One pass: the position of a request is the number of requests ahead of it in its
         * queue, dropped or not, so every request can be decided on its own.
         * Sequentially consistent: the Request Broker takes the requests of a queue in queue
         * order and a dropped request never takes a batch slot (Section 4.1, the broker's
         * drop-or-infer step), so the position is the number of requests ahead that were
         * KEPT; each queue is then a chain of decisions, taken in order.
         * Ranked: in a downstream queue the request does not join the back; it takes the place its
         * budget gives it among the requests queued there now (the queue is kept in budget order,
         * Section 3.3), so the requests ahead of it at stage i are those that queue's order puts
         * before a newcomer with its deadline: deadline <= its own under low budget first (the
         * ones already there win ties), deadline >= its own under high budget first, everybody
         * in arrival order. */
        int64_t* kept = (int64_t*)calloc((size_t)S, sizeof(int64_t));
        #pragma omp parallel for schedule(static) num_threads(nthreads) if (!consistent)
        for (int64_t j = 0; j < m; ++j) {
            int32_t r = q[j].idx;
            int k = clamp_stage(stage[r], S);
            int64_t pos = consistent ? kept[k] : j - qstart[k];   /* requests ahead of r in its own queue */
            int64_t ahead[64];                                    /* S <= 64: requests ahead of r in every other queue */
            for (int i = 0; i < S; ++i) {
                ahead[i] = qlen[i];
                if (!ranked || M[i] == MODE_FCFS) continue;
                ahead[i] = 0;
                for (int64_t t = qstart[i]; t < qstart[i + 1]; ++t) {
                    int32_t other = deadline[q[t].idx];
                    if (M[i] == MODE_HBF ? other >= deadline[r] : other <= deadline[r]) ahead[i] += 1;
                }
            }
            wide_t best = -1;
            if (sub) {
                /* Eq.(4): the Request Broker's own part plus the State Planner's L_sub */
                best = stage_cost(L + (int64_t)k * LAT_ENTRIES, B[k], Wk[k], pos) + (wide_t)sub[(int64_t)u * S + k];
            } else
            for (int64_t p = 0; p < ps.P; ++p) {
                int32_t a = ps.ptr[p], b = ps.ptr[p + 1];
                int32_t at = -1;
                for (int32_t t = a; t < b; ++t) if (ps.stage[t] == k) { at = t; break; }
                if (at < 0) continue;                    /* path does not pass through stage k */
                wide_t sum = stage_cost(L + (int64_t)k * LAT_ENTRIES, B[k], Wk[k], pos);
                for (int32_t t = at + 1; t < b; ++t) {
                    int32_t i = ps.stage[t];
                    sum += stage_cost(L + (int64_t)i * LAT_ENTRIES, B[i], Wk[i], ahead[i]);
                }
                if (sum > best) best = sum;
            }
            wide_t cap = (wide_t)INT32_MAX;
            wide_t finish = (wide_t)now[u] + best;
            est[r] = (int32_t)(best > cap ? cap : best);
            if (finish > cap) finish = cap;
            drop[r] = (uint8_t)(finish > (wide_t)deadline[r]);
            if (consistent && !drop[r]) kept[k] += 1;
        }
        free(kept);
        free(fill);
        free(q);
        free(qstart);
        free(qlen);
        paths_free(&ps);
    }
    seg_ptr[(int64_t)K * S] = snap_ptr[K];
    free(col_base);
    return status;
}

int pard_oracle_estimate_drop(
        int32_t K, int32_t S, int32_t dag_shared,
        const int32_t* row_ptr, const int32_t* col,
        const int32_t* batch, const int32_t* workers, const int32_t* lat, const int32_t* mode,
        int64_t n, const int32_t* arrival, const int32_t* deadline, const int32_t* stage,
        const int32_t* snap_ptr, const int32_t* now,
        int32_t* est, uint8_t* drop, int32_t* order, int32_t* seg_ptr,
        int32_t nthreads) {
    return estimate_drop_impl(K, S, dag_shared, row_ptr, col, batch, workers, lat, mode, n, arrival, deadline, stage,
                              snap_ptr, now, NULL, 0, 0, est, drop, order, seg_ptr, nthreads);
}

/* The same with the downstream part given: est = own-stage cost at the queue position
 * + sub[snapshot * S + stage]  (Eq.(4): Request Broker part + State Planner part). */
int pard_oracle_estimate_drop_sub(
        int32_t K, int32_t S, int32_t dag_shared,
        const int32_t* row_ptr, const int32_t* col,
        const int32_t* batch, const int32_t* workers, const int32_t* lat, const int32_t* mode,
        int64_t n, const int32_t* arrival, const int32_t* deadline, const int32_t* stage,
        const int32_t* snap_ptr, const int32_t* now, const int64_t* sub,
        int32_t* est, uint8_t* drop, int32_t* order, int32_t* seg_ptr,
        int32_t nthreads) {
    return estimate_drop_impl(K, S, dag_shared, row_ptr, col, batch, workers, lat, mode, n, arrival, deadline, stage,
                              snap_ptr, now, sub, 0, 0, est, drop, order, seg_ptr, nthreads);
}

/* Sequentially consistent dropping: as above (sub may be NULL), but a request's position is
 * the number of requests ahead of it in its queue that were kept. */
int pard_oracle_estimate_drop_consistent(
        int32_t K, int32_t S, int32_t dag_shared,
        const int32_t* row_ptr, const int32_t* col,
        const int32_t* batch, const int32_t* workers, const int32_t* lat, const int32_t* mode,
        int64_t n, const int32_t* arrival, const int32_t* deadline, const int32_t* stage,
        const int32_t* snap_ptr, const int32_t* now, const int64_t* sub,
        int32_t* est, uint8_t* drop, int32_t* order, int32_t* seg_ptr,
        int32_t nthreads) {
    return estimate_drop_impl(K, S, dag_shared, row_ptr, col, batch, workers, lat, mode, n, arrival, deadline, stage,
                              snap_ptr, now, sub, 1, 0, est, drop, order, seg_ptr, nthreads);
}

/* Ranked downstream positions: as pard_oracle_estimate_drop, but in every later queue the request
 * counts only the requests that queue's order would serve before it (see the comment in the
 * implementation), not the whole queue. */
int pard_oracle_estimate_drop_ranked(
        int32_t K, int32_t S, int32_t dag_shared,
        const int32_t* row_ptr, const int32_t* col,
        const int32_t* batch, const int32_t* workers, const int32_t* lat, const int32_t* mode,
        int64_t n, const int32_t* arrival, const int32_t* deadline, const int32_t* stage,
        const int32_t* snap_ptr, const int32_t* now,
        int32_t* est, uint8_t* drop, int32_t* order, int32_t* seg_ptr,
        int32_t nthreads) {
    if (S > 64) return 4;
    return estimate_drop_impl(K, S, dag_shared, row_ptr, col, batch, workers, lat, mode, n, arrival, deadline, stage,
                              snap_ptr, now, NULL, 0, 1, est, drop, order, seg_ptr, nthreads);
}

/*
 * Latency of the modules after the current one, per (snapshot, stage): L_sub of Eq.(4),
 * maximum over the downstream DAG paths.
 *
 * For the stages i after stage k on one path, with n_i = qlen[snapshot][i] requests queued:
 *   q_i = floor(ceil(n_i/B_i) * lat_i[B_i] / W_i)     queueing delay (snapshot stand-in for the
 *                                                     monitored average), or, when qdelay is not
 *                                                     NULL, the monitored q_i = max(qdelay[u*S+i], 0)
 *   d_i = lat_i[min(B_i, n_i + 1)]                     execution duration at the batch size a
 *                                                     joining request would see
 *   (with the stand-in, q_i + d_i is stage_cost(n_i), the term the estimate path adds per
 *   downstream stage)
 *
 *   variant 0, full   : sum q_i + sum d_i + w
 *   variant 1, lower  : sum q_i + sum d_i               (batch wait assumed 0)
 *   variant 2, upper  : sum q_i + sum d_i + sum d_i     (batch wait assumed sum d_i)
 *   variant 3, sf     : sum d_i                         (ignores Q and W of later modules)
 *   variant 4, back   : 0                               (preceding and current modules only)
 *
 * w = lambda-quantile (lambda = lam_num/lam_den) of the aggregated batch wait time, sampled:
 * sample j (0 <= j < M) draws, independently for every stage i, one arrival of the collected
 * arrival process, a = max(samples[picks[j*S + i] mod M], 0); a module starts a batch every d_i
 * (batches run back to back, boundaries at multiples of d_i), so that arrival waits
 *   W(j,i) = (d_i - a mod d_i) mod d_i      (0 when d_i = 0)
 * for the next batch; T_j = sum over the path's later stages of W(j,i).  With the T_j sorted
 * ascending, w = T[ceil(lambda*M) - 1]; lambda = 0 gives 0 and lambda = 1 gives sum d_i, the end
 * points the paper states.  The random draws (picks) are inputs, not generated here.
 *
 * Output sub[K*S], saturated at 2^40 microseconds.  Returns 0, or a positive code for a
 * malformed DAG, 4 for bad arguments.
 */
static int cmp_u64(const void* a, const void* b) {
    uint64_t x = *(const uint64_t*)a, y = *(const uint64_t*)b;
    return x < y ? -1 : (x > y ? 1 : 0);
}

int pard_oracle_sub_latency(
        int32_t K, int32_t S, int32_t dag_shared,
        const int32_t* row_ptr, const int32_t* col,
        const int32_t* batch, const int32_t* workers, const int32_t* lat,
        const int32_t* qlen, const int32_t* qdelay,
        int32_t variant, int64_t lam_num, int64_t lam_den,
        int64_t M, const int32_t* samples, const uint32_t* picks,
        int64_t* sub, int32_t nthreads) {
    if (nthreads < 1) nthreads = 1;
    if (variant < 0 || variant > 4) return 4;
    if (variant == 0 && (lam_den <= 0 || lam_num < 0 || lam_num > lam_den || M < 1 || !samples || !picks)) return 4;
    int status = 0;
    int64_t D = dag_shared ? 1 : K;
    int64_t* col_base = (int64_t*)malloc(sizeof(int64_t) * (size_t)(D + 1));
    col_base[0] = 0;
    for (int64_t d = 0; d < D; ++d) col_base[d + 1] = col_base[d] + row_ptr[d * (S + 1) + S];
    const wide_t cap = (wide_t)1 << 40;

    #pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
    for (int32_t u = 0; u < K; ++u) {
        int64_t d = dag_shared ? 0 : u;
        const int32_t* B = batch + d * S;
        const int32_t* Wk = workers + d * S;
        const int32_t* L = lat + d * S * LAT_ENTRIES;
        const int32_t* nq = qlen + (int64_t)u * S;
        paths_t ps;
        int err = enumerate_paths(S, row_ptr + d * (S + 1), col + col_base[d], &ps);
        if (err) {
            #pragma omp critical
            status = err;
            paths_free(&ps);
            continue;
        }
        uint64_t* T = (uint64_t*)malloc(sizeof(uint64_t) * (size_t)(M > 0 ? M : 1));
        for (int k = 0; k < S; ++k) {
            wide_t best = 0;
            for (int64_t p = 0; p < ps.P; ++p) {
                int32_t a = ps.ptr[p], b = ps.ptr[p + 1];
                int32_t at = -1;
                for (int32_t t = a; t < b; ++t) if (ps.stage[t] == k) { at = t; break; }
                if (at < 0) continue;                    /* path does not pass through stage k */
                wide_t sum_qd = 0, sum_d = 0;
                for (int32_t t = at + 1; t < b; ++t) {
                    int32_t i = ps.stage[t];
                    int64_t seen = (int64_t)nq[i] + 1 < B[i] ? (int64_t)nq[i] + 1 : B[i];
                    wide_t d_i = L[(int64_t)i * LAT_ENTRIES + seen - 1];
                    if (qdelay) {
                        int32_t q_i = qdelay[(int64_t)u * S + i];
                        sum_qd += (q_i > 0 ? q_i : 0) + d_i;
                    } else {
                        sum_qd += stage_cost(L + (int64_t)i * LAT_ENTRIES, B[i], Wk[i], nq[i]);
                    }
                    sum_d += d_i;
                }
                wide_t lsub;
                if (variant == 1) lsub = sum_qd;
                else if (variant == 2) lsub = sum_qd + sum_d;
                else if (variant == 3) lsub = sum_d;
                else if (variant == 4) lsub = 0;
                else {
                    wide_t w;
                    if (lam_num == 0) w = 0;
                    else if (lam_num == lam_den) w = sum_d;
                    else {
                        for (int64_t j = 0; j < M; ++j) {
                            uint64_t total = 0;
                            for (int32_t t = at + 1; t < b; ++t) {
                                int32_t i = ps.stage[t];
                                int64_t seen = (int64_t)nq[i] + 1 < B[i] ? (int64_t)nq[i] + 1 : B[i];
                                int64_t di = L[(int64_t)i * LAT_ENTRIES + seen - 1];
                                if (di <= 0) continue;
                                int64_t arr = samples[picks[j * S + i] % (uint64_t)M];
                                if (arr < 0) arr = 0;
                                total += (uint64_t)((di - arr % di) % di);
                            }
                            T[j] = total;
                        }
                        qsort(T, (size_t)M, sizeof(uint64_t), cmp_u64);
                        int64_t rank = (int64_t)(((wide_t)lam_num * M + lam_den - 1) / lam_den);   /* ceil(lambda*M) >= 1 */
                        w = (wide_t)T[rank - 1];
                    }
                    lsub = sum_qd + w;
                }
                if (lsub > best) best = lsub;
            }
            sub[(int64_t)u * S + k] = (int64_t)(best > cap ? cap : best);
        }
        free(T);
        paths_free(&ps);
    }
    free(col_base);
    return status;
}

/*
 * Monitored queueing delay q_i per (snapshot u, stage s): the linearly weighted mean of the
 * recent delay samples inside a sliding window (Section 3.2, State Planner; default window 5 s).
 *
 * Series g = u*S + s holds `len` samples (time[g*len + j], delay[g*len + j]), in any order: a
 * request left the queue at `time` after waiting `delay` there (microseconds).  Seen from
 * now[u], a sample of age = now - time weighs
 *   w = window - age   for 0 <= age < window,   0 otherwise (older than the window, or later than now)
 * so the newest sample counts most and the weight falls linearly to nothing at the window's far
 * edge.  q = floor(sum w * max(delay, 0) / sum w), and 0 when no sample lies in the window.
 * Returns 0, or 4 for bad arguments.
 */
int pard_oracle_queue_delay(
        int32_t K, int32_t S, int32_t len, int64_t window,
        const int32_t* time, const int32_t* delay, const int32_t* now, int32_t* q) {
    if (len < 0 || window < 1) return 4;
    for (int64_t g = 0; g < (int64_t)K * S; ++g) {
        wide_t num = 0, den = 0;
        for (int32_t j = 0; j < len; ++j) {
            wide_t age = (wide_t)now[g / S] - time[g * len + j];
            if (age < 0 || age >= window) continue;
            wide_t w = window - age;
            wide_t x = delay[g * len + j] > 0 ? delay[g * len + j] : 0;
            num += w * x;
            den += w;
        }
        q[g] = den > 0 ? (int32_t)(num / den) : 0;
    }
    return 0;
}

/*
 * Adaptive request priority with delayed transition (Section 3.3).
 *
 * Per (snapshot u, stage s), from the series rate[(u*S+s)*T + t], t = 0..T-1, of the module's
 * monitored input workload T_in (requests per second):
 *   T_m     = W * B / lat[B]                      module throughput (lat in microseconds, so
 *                                                 T_m = W * B * 10^6 / lat[B] requests per second)
 *   T_s[t]  = floor(mean of rate[max(0,t-w+1) .. t])   the workload filtered by a sliding-window
 *                                                 average of width w
 *   eps     = sum_t |rate[t] - T_s[t]| / sum_t rate[t]     (0 when the series sums to 0)
 *   mu[t]   = rate[t] / T_m
 *   mode[t] = HBF if mu[t] > 1 + eps,  LBF if mu[t] < 1 - eps,  otherwise mode[t-1]
 *   mode[-1] = prev_mode[u*S+s] (LBF when prev_mode is NULL)
 * Output: mode[T-1], the priority in force after the series.  Every comparison is evaluated
 * exactly in integers (cross-multiplied); lat[B] = 0 means unbounded throughput, mu = 0.
 * Returns 0, or 4 for bad arguments.
 */
int pard_oracle_priority_modes(
        int32_t K, int32_t S, int32_t dag_shared,
        const int32_t* batch, const int32_t* workers, const int32_t* lat,
        int32_t T, int32_t window, const int32_t* rate, const int32_t* prev_mode, int32_t* mode_out) {
    if (T < 1 || window < 1) return 4;
    for (int64_t g = 0; g < (int64_t)K * S; ++g) {
        int64_t rec = dag_shared ? g % S : g;
        const int32_t* r = rate + g * T;
        wide_t B = batch[rec], W = workers[rec], latB = lat[rec * LAT_ENTRIES + batch[rec] - 1];
        wide_t sum = 0, dev = 0;
        for (int32_t t = 0; t < T; ++t) {
            int32_t lo = t - window + 1 < 0 ? 0 : t - window + 1;
            wide_t win = 0;
            for (int32_t i = lo; i <= t; ++i) win += r[i];
            wide_t ts = win / (t - lo + 1);                       /* floor of the window mean */
            wide_t d = (wide_t)r[t] - ts;
            dev += d < 0 ? -d : d;
            sum += r[t];
        }
        int32_t mode = prev_mode ? prev_mode[g] : MODE_LBF;
        for (int32_t t = 0; t < T; ++t) {
            /* mu > 1 + eps  <=>  rate * lat[B] * sum > W * B * 10^6 * (sum + dev)   (sum > 0)
             * mu < 1 - eps  <=>  rate * lat[B] * sum < W * B * 10^6 * (sum - dev)
             * with sum = 0 (all rates 0): eps = 0 and mu = 0 < 1 */
            wide_t lhs, hi, lo;
            if (sum > 0) {
                lhs = (wide_t)r[t] * latB * sum;
                hi = W * B * 1000000 * (sum + dev);
                lo = W * B * 1000000 * (sum - dev);
            } else {
                lhs = (wide_t)r[t] * latB;
                hi = lo = W * B * 1000000;
            }
            if (lhs > hi) mode = MODE_HBF;
            else if (lhs < lo) mode = MODE_LBF;
        }
        mode_out[g] = mode;
    }
    return 0;
}

/*
 * Survivor compaction: the queues of `order` with dropped requests removed, same
 * order, plus their offsets.  surv_idx has capacity n; entries past surv_ptr[K*S]
 * are left untouched.
 */
int pard_oracle_compact(int32_t K, int32_t S, int64_t n,
                        const int32_t* order, const int32_t* seg_ptr, const uint8_t* drop,
                        int32_t* surv_idx, int32_t* surv_ptr) {
    (void)n;
    int64_t out = 0;
    for (int64_t g = 0; g < (int64_t)K * S; ++g) {
        surv_ptr[g] = (int32_t)out;
        for (int64_t j = seg_ptr[g]; j < seg_ptr[g + 1]; ++j) {
            int32_t r = order[j];
            if (!drop[r]) surv_idx[out++] = r;
        }
    }
    surv_ptr[(int64_t)K * S] = (int32_t)out;
    return 0;
}


/* ---- reactive baselines (Section 5.1, "Baselines") ------------------------------------------
 *
 * Nexus, as the paper describes it: the queue is walked in arrival order with a window as long as the batch
 * size; the walk ends at the first position at which every request inside the window can still meet the
 * budget of the module it waits at, and everything ahead of that position is dropped.  On a snapshot: the
 * queues are given in the order to scan (order/seg_ptr as
 * written by the estimate call; a plan whose stages use arrival order gives the paper's baseline).  For
 * queue (u, s) with batch size B and n requests, the window at position p holds the requests at positions
 * p .. p + w - 1, w = min(B, n - p) (the last windows are cut off by the end of the queue); its requests run
 * as one batch of w, which takes lat[w]; a request can meet the module's budget when that batch ends no
 * later than its deadline, now + lat[w] <= deadline.  first_kept = the first p whose whole window can
 * (n when no window can); the requests at positions before first_kept are dropped, all others kept.
 * Nothing downstream is looked at (the paper says so: later modules' budgets play no part in this policy).
 */
int pard_oracle_nexus_drop(int32_t K, int32_t S, int32_t dag_shared, const int32_t* batch, const int32_t* lat_us,
                           int64_t n, const int32_t* deadline, const int32_t* order, const int32_t* seg_ptr,
                           const int32_t* now, uint8_t* drop_out, int32_t* first_kept_out) {
    if (K < 1 || S < 1 || n < 0) return 1;
    for (int32_t u = 0; u < K; ++u)
        for (int32_t s = 0; s < S; ++s) {
            const int64_t g = (int64_t)u * S + s;
            const int64_t rec = dag_shared ? s : g;
            const int32_t B = batch[rec];
            const int32_t* lat = lat_us + rec * LAT_ENTRIES;
            const int64_t a = seg_ptr[g], len = (int64_t)seg_ptr[g + 1] - a;
            int64_t first = len;
            for (int64_t p = 0; p < len && first == len; ++p) {
                const int64_t w = len - p < B ? len - p : B;
                const wide_t batch_end = (wide_t)now[u] + (wide_t)lat[w - 1];
                int all_meet = 1;
                for (int64_t i = 0; i < w; ++i)
                    if (batch_end > (wide_t)deadline[order[a + p + i]]) all_meet = 0;
                if (all_meet) first = p;
            }
            first_kept_out[g] = (int32_t)first;
            for (int64_t j = 0; j < len; ++j) drop_out[order[a + j]] = j < first ? 1 : 0;
        }
    return 0;
}

/* Clipper++, as the paper describes it: the end-to-end SLO is shared out among the modules in proportion to
 * their execution durations, SLO_k = SLO * d_k / sum_i d_i, and each module decides by its own share; Clipper
 * itself only drops a request whose latency objective has already passed before inference starts.  On a snapshot a
 * request carries the time it was sent (arrival) and its deadline, so SLO = deadline - arrival, and what it
 * has used so far is now - arrival; the time it entered its current module is not known.  The budgets of
 * the modules up to and including the current one add up to SLO * P_k / T_k, where d_i = lat_i[B_i] is a
 * module's execution duration at its batch size, P_k the summed durations from a source to k (k included)
 * and T_k the summed durations of a whole source-to-sink path through k; for a DAG both are taken along the
 * longest such path (P_k = longest way in, T_k = P_k + longest way out).  The request is dropped when it has
 * already used more than that:  now - arrival > SLO * P_k / T_k  (exactly, as rationals: no rounding), which
 * for one module is Clipper's own rule, now > deadline.  T_k = 0 (all durations zero) reads as P_k / T_k = 1.
 */
int pard_oracle_clipper_drop(int32_t K, int32_t S, int32_t dag_shared, const int32_t* dag_row_ptr, const int32_t* dag_col,
                             const int32_t* batch, const int32_t* lat_us, int64_t n, const int32_t* arrival,
                             const int32_t* deadline, const int32_t* stage, const int32_t* snap_ptr, const int32_t* now,
                             uint8_t* drop_out) {
    if (K < 1 || S < 1 || n < 0) return 1;
    const int D = dag_shared ? 1 : K;
    wide_t* way_in = (wide_t*)malloc(sizeof(wide_t) * (size_t)D * (size_t)S);     /* P_k */
    wide_t* whole = (wide_t*)malloc(sizeof(wide_t) * (size_t)D * (size_t)S);      /* T_k */
    int64_t col_base = 0;
    int err = 0;
    for (int d = 0; d < D && !err; ++d) {
        const int32_t* rp = dag_row_ptr + (int64_t)d * (S + 1);
        paths_t ps;
        if (enumerate_paths(S, rp, dag_col + col_base, &ps)) { err = 2; paths_free(&ps); break; }
        col_base += rp[S];
        for (int k = 0; k < S; ++k) {
            wide_t longest_in = -1, longest_out = -1;
            for (int64_t q = 0; q < ps.P; ++q) {
                for (int32_t e = ps.ptr[q]; e < ps.ptr[q + 1]; ++e) {
                    if (ps.stage[e] != k) continue;
                    wide_t in = 0, out = 0;
                    for (int32_t t = ps.ptr[q]; t <= e; ++t) {
                        const int64_t rec = (int64_t)d * S + ps.stage[t];
                        in += lat_us[rec * LAT_ENTRIES + batch[rec] - 1];
                    }
                    for (int32_t t = e + 1; t < ps.ptr[q + 1]; ++t) {
                        const int64_t rec = (int64_t)d * S + ps.stage[t];
                        out += lat_us[rec * LAT_ENTRIES + batch[rec] - 1];
                    }
                    if (in > longest_in) longest_in = in;
                    if (out > longest_out) longest_out = out;
                }
            }
            way_in[(int64_t)d * S + k] = longest_in;
            whole[(int64_t)d * S + k] = longest_in + longest_out;
        }
        paths_free(&ps);
    }
    for (int32_t u = 0; u < K && !err; ++u)
        for (int64_t r = snap_ptr[u]; r < snap_ptr[u + 1]; ++r) {
            const int k = clamp_stage(stage[r], S);
            const int64_t rec = (int64_t)(dag_shared ? 0 : u) * S + k;
            const wide_t used = (wide_t)now[u] - (wide_t)arrival[r];
            const wide_t slo = (wide_t)deadline[r] - (wide_t)arrival[r];
            if (whole[rec] == 0) drop_out[r] = used > slo ? 1 : 0;
            else drop_out[r] = used * whole[rec] > slo * way_in[rec] ? 1 : 0;
        }
    free(way_in);
    free(whole);
    return err;
}
