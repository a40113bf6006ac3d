/*
 * CPU ORACLE -- test infrastructure only.
 *
 * Plain, slow, step-by-step implementation of what the GPU library computes:
 *   - the offline Minimizing Makespan Bin Packing (MMBP) model of the paper's section
 *     "Offline requests scheduling & theoretical lower bound" (objective min max_j t_j,
 *     every request on exactly one client, t_j >= sum of the T_i assigned to client j),
 *     searched by best-improvement over the full move + swap neighbourhood;
 *   - the theoretical lower bound T^LB = t^p* + t^d* of the same section, with t^d* replaced
 *     by the classical relaxation bounds of the makespan problem;
 *   - the online iteration scheduling rule of section "Online requests and iteration
 *     scheduling" (compare prefill cost C_p with waited decode time C_d; C_p >= C_d keeps
 *     decoding), stepped one iteration at a time with the affine time model of section
 *     "Experiment settings and baseline".
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call this file.
 * It shares no code, header, table or helper with the HIP sources.
 *
 * Pins (see tests): candidate values against a from-scratch recomputation of every load;
 * selection / tie-break against hand-worked examples; result quality against brute-force
 * enumeration of all assignments; bounds and simulator against closed forms and the
 * paper's two worked time-model examples.  The meaning given to C_d (decode time
 * accumulated since the last prefill) is a reading of an ambiguous passage: the decision
 * rule is "parity unpinned" with respect to the paper (no trace is published).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ST_OK 0
#define ST_TRUNCATED 1
#define ST_BAD_ASSIGN 2
#define ST_BAD_COST 3
#define ST_BAD_SIM_INPUT 4

#define COST_SUM_LIMIT ((int64_t)1 << 62)

static int64_t max2(int64_t a, int64_t b) { return a > b ? a : b; }

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------------------------
 * Local search, one scenario.
 * Candidate value = makespan of the assignment after applying the candidate:
 *   move (i -> b):   loads change on a = assign[i] and b:  load[a] - T_i, load[b] + T_i
 *   swap (i <-> k):  with d = T_i - T_k:                    load[a] - d,   load[b] + d
 * and every other client keeps its load, so the makespan is the max of the two new loads and
 * of the largest untouched load (objective of the MMBP model).
 * ids: move = i*M + b ; swap = N*M + i*N + k (i < k).  Best = smallest (value, id).
 * ------------------------------------------------------------------------------------------ */
typedef struct { int64_t value; uint64_t id; int valid; } best_t;

static void best_take(best_t *b, int64_t value, uint64_t id)
{
    if (!b->valid || value < b->value || (value == b->value && id < b->id)) {
        b->value = value; b->id = id; b->valid = 1;
    }
}

static void ls_one(const int64_t *cost, int N, int M, int cap, int max_passes, int32_t *assign,
                   int64_t *load, int64_t *makespan, int32_t *passes_out, uint64_t *evals_out,
                   uint64_t *applied_log, int32_t *status, int inner_parallel)
{
    int32_t *cnt = (int32_t *)calloc((size_t)M, sizeof(int32_t));
    int64_t *others = (int64_t *)malloc((size_t)M * M * sizeof(int64_t));
    uint64_t evals = 0;
    int passes = 0;
    int st = ST_OK;

    for (int j = 0; j < M; j++) load[j] = 0;
    *makespan = 0; *passes_out = 0; if (evals_out) *evals_out = 0;

    /* validation */
    int bad_cost = 0, bad_assign = 0;
    int64_t total = 0;
    for (int i = 0; i < N; i++) {
        if (cost[i] < 0) { bad_cost = 1; break; }
        if (cost[i] >= COST_SUM_LIMIT || total + cost[i] >= COST_SUM_LIMIT) { bad_cost = 1; break; }
        total += cost[i];
    }
    for (int i = 0; i < N; i++) {
        if (assign[i] < 0 || assign[i] >= M) { bad_assign = 1; break; }
        cnt[assign[i]]++;
    }
    if (!bad_assign)
        for (int j = 0; j < M; j++) if (cnt[j] > cap) bad_assign = 1;
    if (bad_cost || bad_assign) {
        *status = bad_cost ? ST_BAD_COST : ST_BAD_ASSIGN;
        free(cnt); free(others);
        return;
    }
    for (int i = 0; i < N; i++) load[assign[i]] += cost[i];

    for (;;) {
        if (passes == max_passes) { st = ST_TRUNCATED; break; }
        int64_t T = 0;
        for (int j = 0; j < M; j++) T = max2(T, load[j]);
        /* largest load among clients other than a and b, by definition */
        for (int a = 0; a < M; a++)
            for (int b = 0; b < M; b++) {
                int64_t o = 0;
                for (int j = 0; j < M; j++) if (j != a && j != b) o = max2(o, load[j]);
                others[(size_t)a * M + b] = o;
            }
        best_t best = {0, 0, 0};
        /* moves */
        for (int i = 0; i < N; i++) {
            int a = assign[i];
            for (int b = 0; b < M; b++) {
                if (b == a) continue;
                evals++;
                if (cnt[b] + 1 > cap) continue;
                int64_t v = max2(max2(load[a] - cost[i], load[b] + cost[i]), others[(size_t)a * M + b]);
                best_take(&best, v, (uint64_t)i * (uint64_t)M + (uint64_t)b);
            }
        }
        /* swaps: one loop for both ways of running it.  With inner_parallel the rows i are
         * dealt to the threads of a team and the per-thread bests are merged with the same
         * (value, id) order, which is total, so the result does not depend on the split; without
         * it the team has one thread and the loop runs as written. */
        uint64_t swap_evals = 0;
#pragma omp parallel if (inner_parallel)
        {
            best_t mine = {0, 0, 0};
            uint64_t my_evals = 0;
#pragma omp for schedule(dynamic, 64) nowait
            for (int i = 0; i < N; i++) {
                int a = assign[i];
                for (int k = i + 1; k < N; k++) {
                    int b = assign[k];
                    if (a == b) continue;
                    my_evals++;
                    int64_t d = cost[i] - cost[k];
                    int64_t v = max2(max2(load[a] - d, load[b] + d), others[(size_t)a * M + b]);
                    best_take(&mine, v, (uint64_t)N * M + (uint64_t)i * N + (uint64_t)k);
                }
            }
#pragma omp critical
            {
                swap_evals += my_evals;
                if (mine.valid) best_take(&best, mine.value, mine.id);
            }
        }
        evals += swap_evals;
        if (!best.valid || best.value >= T) { st = ST_OK; break; }
        /* apply */
        uint64_t NM = (uint64_t)N * (uint64_t)M;
        if (best.id < NM) {
            int i = (int)(best.id / (uint64_t)M), b = (int)(best.id % (uint64_t)M);
            int a = assign[i];
            load[a] -= cost[i]; load[b] += cost[i];
            cnt[a]--; cnt[b]++;
            assign[i] = b;
        } else {
            uint64_t r = best.id - NM;
            int i = (int)(r / (uint64_t)N), k = (int)(r % (uint64_t)N);
            int a = assign[i], b = assign[k];
            int64_t d = cost[i] - cost[k];
            load[a] -= d; load[b] += d;
            assign[i] = b; assign[k] = a;
        }
        if (applied_log) applied_log[passes] = best.id;
        passes++;
    }
    int64_t T = 0;
    for (int j = 0; j < M; j++) T = max2(T, load[j]);
    *makespan = T;
    *passes_out = passes;
    if (evals_out) *evals_out = evals;
    *status = st;
    free(cnt); free(others);
}

/* mode: 0 = threads over scenarios (each scenario's scan serial), 1 = scenarios one after the
 * other, threads inside the swap scan, -1 = pick by batch size.  Results do not depend on it. */
int oracle_local_search_mode(const int64_t *cost, int S, int N, int M, int cap, int max_passes,
                             int32_t *assign, int64_t *load_out, int64_t *makespan_out,
                             int32_t *passes_out, uint64_t *evals_out, uint64_t *applied_log,
                             int32_t *status_out, int mode)
{
    if (!cost || !assign || !load_out || !makespan_out || !passes_out || !status_out) return -1;
    if (S <= 0 || N <= 0 || M <= 0 || cap <= 0 || max_passes < 0) return -1;
    if (mode < -1 || mode > 1) return -1;
    if ((int64_t)N > (int64_t)M * cap) return -2;
    int threads = oracle_num_threads();
    int inner = mode >= 0 ? mode : !(S >= threads || threads == 1);
#pragma omp parallel for schedule(dynamic, 1) if (!inner)
    for (int s = 0; s < S; s++)
        ls_one(cost + (size_t)s * N, N, M, cap, max_passes, assign + (size_t)s * N,
               load_out + (size_t)s * M, makespan_out + s, passes_out + s,
               evals_out ? evals_out + s : 0,
               applied_log ? applied_log + (size_t)s * max_passes : 0, status_out + s, inner);
    return 0;
}

int oracle_local_search(const int64_t *cost, int S, int N, int M, int cap, int max_passes,
                        int32_t *assign, int64_t *load_out, int64_t *makespan_out,
                        int32_t *passes_out, uint64_t *evals_out, uint64_t *applied_log,
                        int32_t *status_out)
{
    return oracle_local_search_mode(cost, S, N, M, cap, max_passes, assign, load_out, makespan_out,
                                    passes_out, evals_out, applied_log, status_out, -1);
}

/* ------------------------------------------------------------------------------------------
 * Brute force: optimum of the MMBP model (with the cardinality limit) over all M^N
 * assignments.  Tiny instances only.
 * ------------------------------------------------------------------------------------------ */
static void bf_rec(const int64_t *cost, int N, int M, int cap, int i, int64_t *load, int32_t *cnt,
                   int64_t *best)
{
    if (i == N) {
        int64_t T = 0;
        for (int j = 0; j < M; j++) T = max2(T, load[j]);
        if (*best < 0 || T < *best) *best = T;
        return;
    }
    for (int j = 0; j < M; j++) {
        if (cnt[j] + 1 > cap) continue;
        cnt[j]++; load[j] += cost[i];
        bf_rec(cost, N, M, cap, i + 1, load, cnt, best);
        cnt[j]--; load[j] -= cost[i];
    }
}

/* returns the optimum makespan, or -1 if no feasible assignment exists */
int64_t oracle_brute_force_opt(const int64_t *cost, int N, int M, int cap)
{
    int64_t *load = (int64_t *)calloc((size_t)M, sizeof(int64_t));
    int32_t *cnt = (int32_t *)calloc((size_t)M, sizeof(int32_t));
    int64_t best = -1;
    bf_rec(cost, N, M, cap, 0, load, cnt, &best);
    free(load); free(cnt);
    return best;
}

/* ------------------------------------------------------------------------------------------
 * Lower bound.  T^LB = t^p* + t^d*  (paper, theoretical lower bound equation).
 *   t^d*: the optimum of the MMBP model is bounded below by
 *           L1 = ceil(sum T_i / M), L2 = largest T_i,
 *           L3 = T_(M) + T_(M+1) (descending order; two of the M+1 largest share a client)
 *   t^p*: T^p_L * floor(sum N^p_i / N^cap_L) when the caller supplies prefill tokens.
 * ------------------------------------------------------------------------------------------ */
static int cmp_desc(const void *x, const void *y)
{
    int64_t a = *(const int64_t *)x, b = *(const int64_t *)y;
    return a < b ? 1 : (a > b ? -1 : 0);
}

int oracle_lower_bound(const int64_t *cost, int S, int N, int M, const int32_t *prefill_tokens,
                       int64_t ncap_L, int64_t tp_L, int64_t *lb_out, int32_t *status_out)
{
    if (!cost || !lb_out || !status_out || S <= 0 || N <= 0 || M <= 0) return -1;
#pragma omp parallel for schedule(static)
    for (int s = 0; s < S; s++) {
        const int64_t *c = cost + (size_t)s * N;
        int64_t *sorted = (int64_t *)malloc((size_t)N * sizeof(int64_t));
        int bad = 0;
        int64_t sum = 0;
        for (int i = 0; i < N; i++) {
            if (c[i] < 0 || c[i] >= COST_SUM_LIMIT || sum + c[i] >= COST_SUM_LIMIT) { bad = 1; break; }
            sum += c[i];
        }
        /* N^p_i is a token count: a negative entry makes the scenario's input invalid */
        if (prefill_tokens && ncap_L > 0)
            for (int i = 0; i < N; i++) if (prefill_tokens[(size_t)s * N + i] < 0) bad = 1;
        if (bad) { lb_out[s] = 0; status_out[s] = ST_BAD_COST; free(sorted); continue; }
        memcpy(sorted, c, (size_t)N * sizeof(int64_t));
        qsort(sorted, (size_t)N, sizeof(int64_t), cmp_desc);
        int64_t L1 = (sum + M - 1) / M;
        int64_t L2 = sorted[0];
        int64_t L3 = (N >= M + 1) ? sorted[M - 1] + sorted[M] : 0;
        int64_t lbd = max2(L1, max2(L2, L3));
        int64_t lbp = 0;
        if (prefill_tokens && ncap_L > 0) {
            int64_t tok = 0;
            for (int i = 0; i < N; i++) tok += prefill_tokens[(size_t)s * N + i];
            lbp = tp_L * (tok / ncap_L);
        }
        lb_out[s] = lbd + lbp;
        status_out[s] = ST_OK;
        free(sorted);
    }
    return 0;
}

/* ------------------------------------------------------------------------------------------
 * Longest-processing-time start for the MMBP model (min max_j t_j with at most cap requests per
 * client): take the requests by decreasing cost T_i (equal costs: lower index first) and give
 * each to the client with the smallest load t_j among those that still have room (equal loads:
 * lower client index).  The classical list-scheduling rule; with cap >= N its makespan is at
 * most (4/3 - 1/(3M)) times the optimum.
 * order_out (nullable) receives the request indices in the order they were taken.
 * ------------------------------------------------------------------------------------------ */
typedef struct { int64_t cost; int32_t idx; } lpt_item;

static int cmp_lpt(const void *x, const void *y)
{
    const lpt_item *a = (const lpt_item *)x, *b = (const lpt_item *)y;
    if (a->cost != b->cost) return a->cost < b->cost ? 1 : -1;
    return a->idx < b->idx ? -1 : (a->idx > b->idx ? 1 : 0);
}

int oracle_lpt_start(const int64_t *cost, int S, int N, int M, int cap, int32_t *assign_out,
                     int64_t *load_out, int32_t *order_out, int32_t *status_out)
{
    if (!cost || !assign_out || !load_out || !status_out || S <= 0 || N <= 0 || M <= 0 || cap <= 0) return -1;
    if ((int64_t)N > (int64_t)M * cap) return -2;
#pragma omp parallel for schedule(dynamic, 1)
    for (int s = 0; s < S; s++) {
        const int64_t *c = cost + (size_t)s * N;
        int32_t *asg = assign_out + (size_t)s * N;
        int64_t *load = load_out + (size_t)s * M;
        for (int j = 0; j < M; j++) load[j] = 0;
        int bad = 0;
        int64_t sum = 0;
        for (int i = 0; i < N; i++) {
            if (c[i] < 0 || c[i] >= COST_SUM_LIMIT || sum + c[i] >= COST_SUM_LIMIT) { bad = 1; break; }
            sum += c[i];
        }
        if (bad) {
            status_out[s] = ST_BAD_COST;
            for (int i = 0; i < N; i++) { asg[i] = -1; if (order_out) order_out[(size_t)s * N + i] = -1; }
            continue;
        }
        lpt_item *it = (lpt_item *)malloc((size_t)N * sizeof(lpt_item));
        int32_t *cnt = (int32_t *)calloc((size_t)M, sizeof(int32_t));
        for (int i = 0; i < N; i++) { it[i].cost = c[i]; it[i].idx = i; }
        qsort(it, (size_t)N, sizeof(lpt_item), cmp_lpt);
        for (int q = 0; q < N; q++) {
            int best = -1;
            for (int j = 0; j < M; j++) {
                if (cnt[j] >= cap) continue;
                if (best < 0 || load[j] < load[best]) best = j;
            }
            /* N <= M*cap: some client has room */
            asg[it[q].idx] = best;
            load[best] += it[q].cost;
            cnt[best]++;
            if (order_out) order_out[(size_t)s * N + q] = it[q].idx;
        }
        status_out[s] = ST_OK;
        free(it); free(cnt);
    }
    return 0;
}

/* ------------------------------------------------------------------------------------------
 * Extended lower bound.  Same equation T^LB = t^p* + t^d*, with more relaxation bounds on t^d*
 * and a level table for t^p* (levels l with token capacity N^cap_l and prefill time T^p_l, as in
 * the paper's prefill-length constraints).
 *   L1, L2 as above.
 *   L3(k) = T_(kM+1) + T_(kM) + ... + T_(kM+1-k)   (descending order, k >= 1, kM+1 <= N):
 *           of the kM+1 largest requests some client holds at least k+1, and those cost at least
 *           as much as the k+1 smallest of them.  Taken over k <= kmax (kmax <= 0: no limit of the
 *           caller's) with kM+1 <= rank_limit (the library's own limit on the ranks it looks at;
 *           any subset of the k gives a valid bound).  L3 = max_k L3(k), k3 = the smallest k that
 *           attains it (0 when no k qualifies).
 *   Lcap  per-client cardinality limits cap[j] (nullable): client j holds at least
 *           n_j = max(0, N - sum_{j' != j} cap[j']) requests, so its load is at least the sum of
 *           the n_j smallest costs; Lcap = that sum for the largest n_j.
 *   t^p*  tp_form 0: the paper's floor form on the level L of largest capacity (among equal
 *           capacities the smaller time), T^p_L * floor(sum N^p_i / N^cap_L);
 *         tp_form 1: every prefill stage of level l takes T^p_l for at most N^cap_l tokens, so
 *           any set of stages that covers all tokens takes at least
 *           ceil(sum N^p_i * min_l (T^p_l / N^cap_l))  (valid for every table, whereas the floor
 *           form assumes the largest level is also the most efficient one).
 * parts_out[s] = { L1, L2, L3, k3, Lcap, t^p* }.  lb = max(L1, L2, L3, Lcap) + t^p*.
 * Returns -1 bad argument, -2 if sum cap[j] < N.  Status BAD_COST: invalid cost, negative token
 * count, or t^p* not below 2^62.
 * ------------------------------------------------------------------------------------------ */
int oracle_lower_bound_ex(const int64_t *cost, int S, int N, int M, const int32_t *cap, int kmax,
                          int rank_limit, const int32_t *prefill_tokens, int n_levels,
                          const int64_t *ncap, const int64_t *tp, int tp_form, int64_t *lb_out,
                          int64_t *parts_out, int32_t *status_out)
{
    if (!cost || !lb_out || !status_out || S <= 0 || N <= 0 || M <= 0) return -1;
    if (n_levels < 0 || (n_levels > 0 && (!ncap || !tp)) || (tp_form != 0 && tp_form != 1)) return -1;
    if (rank_limit < 1) return -1;
    for (int l = 0; l < n_levels; l++)
        if (ncap[l] < 1 || ncap[l] > INT32_MAX || tp[l] < 0 || tp[l] > INT32_MAX) return -1;
    int nstar = 0;                                   /* largest n_j */
    if (cap) {
        int64_t capsum = 0;
        for (int j = 0; j < M; j++) { if (cap[j] < 0) return -1; capsum += cap[j]; }
        if (capsum < N) return -2;
        for (int j = 0; j < M; j++) {
            int64_t nj = (int64_t)N - (capsum - cap[j]);
            if (nj > nstar) nstar = (int)nj;
        }
    }
#pragma omp parallel for schedule(static)
    for (int s = 0; s < S; s++) {
        const int64_t *c = cost + (size_t)s * N;
        int64_t *parts = parts_out ? parts_out + (size_t)s * 6 : 0;
        if (parts) for (int q = 0; q < 6; q++) parts[q] = 0;
        int bad = 0;
        int64_t sum = 0, tok = 0;
        for (int i = 0; i < N; i++) {
            if (c[i] < 0 || c[i] >= COST_SUM_LIMIT || sum + c[i] >= COST_SUM_LIMIT) { bad = 1; break; }
            sum += c[i];
        }
        const int with_tp = prefill_tokens && n_levels > 0;
        if (with_tp)
            for (int i = 0; i < N; i++) {
                if (prefill_tokens[(size_t)s * N + i] < 0) bad = 1;
                else tok += prefill_tokens[(size_t)s * N + i];
            }
        /* t^p* */
        int64_t tps = 0;
        if (!bad && with_tp) {
            if (tp_form == 0) {
                int L = 0;
                for (int l = 1; l < n_levels; l++)
                    if (ncap[l] > ncap[L] || (ncap[l] == ncap[L] && tp[l] < tp[L])) L = l;
                int64_t q = tok / ncap[L];
                if (tp[L] > 0 && q > (COST_SUM_LIMIT - 1) / tp[L]) bad = 1;
                else tps = tp[L] * q;
            } else {
                /* min over levels of ceil(tok * tp / ncap), each as q*tp + ceil(r*tp/ncap) */
                for (int l = 0; l < n_levels; l++) {
                    int64_t q = tok / ncap[l], r = tok % ncap[l];
                    if (tp[l] > 0 && q > (COST_SUM_LIMIT - 1) / tp[l] - 1) { bad = 1; break; }
                    int64_t v = q * tp[l] + (r * tp[l] + ncap[l] - 1) / ncap[l];
                    if (l == 0 || v < tps) tps = v;
                }
            }
        }
        if (bad) { lb_out[s] = 0; status_out[s] = ST_BAD_COST; continue; }
        int64_t *sorted = (int64_t *)malloc((size_t)N * sizeof(int64_t));
        memcpy(sorted, c, (size_t)N * sizeof(int64_t));
        qsort(sorted, (size_t)N, sizeof(int64_t), cmp_desc);
        int64_t L1 = (sum + M - 1) / M;
        int64_t L2 = sorted[0];
        int64_t L3 = 0; int k3 = 0;
        for (int k = 1; (int64_t)k * M + 1 <= N && (int64_t)k * M + 1 <= rank_limit; k++) {
            if (kmax > 0 && k > kmax) break;
            int64_t v = 0;
            for (int h = 0; h <= k; h++) v += sorted[(size_t)k * M + 1 - h - 1];   /* rank r is sorted[r-1] */
            if (v > L3) { L3 = v; k3 = k; }
        }
        int64_t Lcap = 0;
        for (int q = 0; q < nstar; q++) Lcap += sorted[N - 1 - q];                   /* the nstar smallest */
        int64_t lbd = max2(max2(L1, L2), max2(L3, Lcap));
        lb_out[s] = lbd + tps;
        status_out[s] = ST_OK;
        if (parts) { parts[0] = L1; parts[1] = L2; parts[2] = L3; parts[3] = k3; parts[4] = Lcap; parts[5] = tps; }
        free(sorted);
    }
    return 0;
}

/* brute force with per-client cardinality limits cap[j] */
static void bf_rec_caps(const int64_t *cost, int N, int M, const int32_t *cap, int i, int64_t *load, int32_t *cnt,
                        int64_t *best)
{
    if (i == N) {
        int64_t T = 0;
        for (int j = 0; j < M; j++) T = max2(T, load[j]);
        if (*best < 0 || T < *best) *best = T;
        return;
    }
    for (int j = 0; j < M; j++) {
        if (cnt[j] + 1 > cap[j]) continue;
        cnt[j]++; load[j] += cost[i];
        bf_rec_caps(cost, N, M, cap, i + 1, load, cnt, best);
        cnt[j]--; load[j] -= cost[i];
    }
}

int64_t oracle_brute_force_opt_caps(const int64_t *cost, int N, int M, const int32_t *cap)
{
    int64_t *load = (int64_t *)calloc((size_t)M, sizeof(int64_t));
    int32_t *cnt = (int32_t *)calloc((size_t)M, sizeof(int32_t));
    int64_t best = -1;
    bf_rec_caps(cost, N, M, cap, 0, load, cnt, &best);
    free(load); free(cnt);
    return best;
}

/* ------------------------------------------------------------------------------------------
 * FNV-1a, 64 bit (published constants: offset basis 0xcbf29ce484222325, prime 0x100000001b3).
 * ------------------------------------------------------------------------------------------ */
uint64_t oracle_fnv1a64(const uint8_t *bytes, size_t n, uint64_t h)
{
    for (size_t i = 0; i < n; i++) { h ^= bytes[i]; h *= 0x100000001b3ULL; }
    return h;
}
uint64_t oracle_fnv1a64_init(void) { return 0xcbf29ce484222325ULL; }

/* ------------------------------------------------------------------------------------------
 * Online iteration simulator, one scenario, one iteration at a time.
 * Iteration kinds: 0 DECODE, 1 PREFILL, 2 IDLE.
 * Canonical trace record (24 bytes, little endian): kind u32, count u32, t_start i64, x i64
 *   PREFILL: count = |A|, x = P (tokens);  IDLE: count = 1, x = 0;
 *   DECODE : maximal run of consecutive decode iterations with equal D: count = run length,
 *            t_start = start of the first, x = D.
 * ------------------------------------------------------------------------------------------ */
typedef struct {
    int32_t cap;
    int32_t policy;             /* 0: the paper's rule; 1: prefill first; 2: prefill first, one request per prefill */
    int64_t a_prefill, b_decode, c_prefill, c_decode;
    int64_t max_prefill_tokens; /* <= 0: unlimited */
} oracle_sim_params;

typedef struct { uint32_t kind, count; int64_t t_start, x; } trace_rec;

typedef struct {
    uint64_t hash;
    trace_rec *buf; int cap; int len;     /* optional record buffer */
    trace_rec run; int run_open;          /* pending decode run */
} trace_t;

static void trace_emit(trace_t *tr, trace_rec r)
{
    uint8_t b[24];
    for (int i = 0; i < 4; i++) b[i] = (uint8_t)(r.kind >> (8 * i));
    for (int i = 0; i < 4; i++) b[4 + i] = (uint8_t)(r.count >> (8 * i));
    for (int i = 0; i < 8; i++) b[8 + i] = (uint8_t)((uint64_t)r.t_start >> (8 * i));
    for (int i = 0; i < 8; i++) b[16 + i] = (uint8_t)((uint64_t)r.x >> (8 * i));
    tr->hash = oracle_fnv1a64(b, 24, tr->hash);
    if (tr->buf && tr->len < tr->cap) tr->buf[tr->len] = r;
    tr->len++;
}
static void trace_flush(trace_t *tr)
{
    if (tr->run_open) { trace_emit(tr, tr->run); tr->run_open = 0; }
}
static void trace_decode(trace_t *tr, int64_t t_start, int64_t D)
{
    if (tr->run_open && tr->run.x == D) { tr->run.count++; return; }
    trace_flush(tr);
    tr->run.kind = 0; tr->run.count = 1; tr->run.t_start = t_start; tr->run.x = D; tr->run_open = 1;
}
static void trace_other(trace_t *tr, uint32_t kind, uint32_t count, int64_t t_start, int64_t x)
{
    trace_flush(tr);
    trace_rec r = {kind, count, t_start, x};
    trace_emit(tr, r);
}

static void sim_one(const int64_t *arrival, const int32_t *in_len, const int32_t *out_len, int N,
                    const oracle_sim_params *p, int64_t *finish, int64_t *total_us,
                    int64_t *busy_slot_us, int32_t *n_prefill_iter, int32_t *n_decode_iter,
                    uint64_t *trace_hash, trace_rec *trace_buf, int trace_capacity,
                    int32_t *trace_len, int32_t *status)
{
    for (int i = 0; i < N; i++) finish[i] = 0;
    *total_us = 0; *busy_slot_us = 0; *n_prefill_iter = 0; *n_decode_iter = 0; *trace_hash = 0;
    if (trace_len) *trace_len = 0;
    for (int i = 0; i < N; i++) {
        if (arrival[i] < 0 || in_len[i] < 1 || out_len[i] < 1 || (i > 0 && arrival[i] < arrival[i - 1])) {
            *status = ST_BAD_SIM_INPUT;
            return;
        }
    }
    int cap = p->cap;
    int32_t *run_id = (int32_t *)malloc((size_t)cap * sizeof(int32_t));   /* running set R */
    int32_t *run_rem = (int32_t *)malloc((size_t)cap * sizeof(int32_t));
    int nR = 0, next = 0, done = 0;
    int64_t t = 0, Cd = 0, busy = 0;
    int32_t npre = 0, ndec = 0;
    trace_t tr; memset(&tr, 0, sizeof tr);
    tr.hash = oracle_fnv1a64_init(); tr.buf = trace_buf; tr.cap = trace_capacity;

    while (done < N) {
        /* admissible set A: longest prefix of the arrived waiting requests that fits the free
         * slots and the prefill token cap (a single oversized head request is still admitted) */
        int free_slots = cap - nR;
        int nA = 0; int64_t P = 0;
        while (next + nA < N && arrival[next + nA] <= t && nA < free_slots) {
            int64_t tok = in_len[next + nA];
            if (p->max_prefill_tokens > 0 && P + tok > p->max_prefill_tokens) {
                if (nA == 0) { P = tok; nA = 1; }
                break;
            }
            P += tok; nA++;
        }
        if (p->policy == 2 && nA > 1) { nA = 1; P = in_len[next]; }   /* baseline without batched prefill */
        if (nA == 0 && nR == 0) {           /* IDLE: jump to the next arrival */
            trace_other(&tr, 2, 1, t, 0);
            t = arrival[next];
            continue;
        }
        int do_prefill;
        if (nA == 0) do_prefill = 0;
        else if (p->policy != 0) do_prefill = 1;      /* baseline: a waiting request is prefilled at once */
        else {
            int64_t Cp = p->a_prefill * P + p->c_prefill;
            if (nR == 0) do_prefill = 1;          /* nothing to decode: forced prefill */
            else if (Cp >= Cd) do_prefill = 0;    /* C_p >= C_d: keep decoding */
            else do_prefill = 1;
        }
        if (do_prefill) {
            int64_t dt = p->a_prefill * P + p->c_prefill;
            trace_other(&tr, 1, (uint32_t)nA, t, P);
            t += dt;
            for (int q = 0; q < nA; q++) { run_id[nR] = next + q; run_rem[nR] = out_len[next + q]; nR++; }
            next += nA;
            busy += (int64_t)nA * dt;
            Cd = 0;
            npre++;
        } else {
            int64_t D = nR;
            int64_t dt = p->b_decode * D + p->c_decode;
            trace_decode(&tr, t, D);
            t += dt;
            int w = 0;
            for (int q = 0; q < nR; q++) {
                run_rem[q] -= 1;
                if (run_rem[q] == 0) { finish[run_id[q]] = t; done++; }
                else { run_id[w] = run_id[q]; run_rem[w] = run_rem[q]; w++; }
            }
            nR = w;
            busy += D * dt;
            Cd += p->b_decode * D;
            ndec++;
        }
    }
    trace_flush(&tr);
    *total_us = t; *busy_slot_us = busy; *n_prefill_iter = npre; *n_decode_iter = ndec;
    *trace_hash = tr.hash;
    if (trace_len) *trace_len = tr.len;
    *status = ST_OK;
    free(run_id); free(run_rem);
}

int oracle_online_iter_sim(const int64_t *arrival_us, const int32_t *in_len, const int32_t *out_len,
                           int S, int N, const oracle_sim_params *p, int64_t *finish_us,
                           int64_t *total_us, int64_t *busy_slot_us, int32_t *n_prefill_iter,
                           int32_t *n_decode_iter, uint64_t *trace_hash, void *trace_buf,
                           int32_t *trace_len, int trace_scenarios, int trace_capacity,
                           int32_t *status_out)
{
    if (!arrival_us || !in_len || !out_len || !p || !finish_us || !total_us || !busy_slot_us ||
        !n_prefill_iter || !n_decode_iter || !trace_hash || !status_out) return -1;
    if (S <= 0 || N <= 0 || p->cap <= 0 || p->policy < 0 || p->policy > 2) return -1;
    if (p->a_prefill < 0 || p->b_decode < 0 || p->c_prefill < 0 || p->c_decode < 0) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int s = 0; s < S; s++) {
        int traced = trace_buf && s < trace_scenarios;
        sim_one(arrival_us + (size_t)s * N, in_len + (size_t)s * N, out_len + (size_t)s * N, N, p,
                finish_us + (size_t)s * N, total_us + s, busy_slot_us + s, n_prefill_iter + s,
                n_decode_iter + s, trace_hash + s,
                traced ? (trace_rec *)trace_buf + (size_t)s * trace_capacity : 0,
                traced ? trace_capacity : 0, (trace_len && s < trace_scenarios) ? trace_len + s : 0,
                status_out + s);
    }
    return 0;
}

/* ------------------------------------------------------------------------------------------
 * Iteration simulator fed by an offline assignment: the "Sorting and Online Preemptive Method"
 * of the paper's section "Online requests and iteration scheduling".
 *   I_j = requests assigned to client j, sorted by N^p_i + N^d_i, longest first (equal lengths:
 *         lower request index first);  remain_token(j) = sum of N^p_i + N^d_i over what is left in I_j.
 *   At an iteration boundary the clients are visited in index order; an idle client takes the
 *   head of its own I_j if there is one, otherwise the head of the I_v of the client v with the
 *   largest remain_token (v lowest among equals), provided that is positive; remain_token of the
 *   queue the request came from is reduced by its length.
 * All requests are known at t = 0 (the algorithm works on the offline request set).  The requests
 * picked at a boundary form the prefill that could be dispatched: C_p = a*P + c_p over their
 * input tokens, limited by the prefill token cap like the FCFS prefix (the first pick always
 * fits), and the policy decides as in the FCFS simulator; picks are only taken when the prefill
 * is dispatched.  Trace, times and counters as in the FCFS simulator.
 * ------------------------------------------------------------------------------------------ */
static void sim_assigned_one(const int32_t *in_len, const int32_t *out_len, const int32_t *assign, int N,
                             const oracle_sim_params *p, int64_t *finish, int64_t *total_us,
                             int64_t *busy_slot_us, int32_t *n_prefill_iter, int32_t *n_decode_iter,
                             uint64_t *trace_hash, int32_t *served_by, int64_t *start_us, trace_rec *trace_buf,
                             int trace_capacity, int32_t *trace_len, int32_t *status)
{
    int cap = p->cap;
    for (int i = 0; i < N; i++) { finish[i] = 0; if (served_by) served_by[i] = -1; if (start_us) start_us[i] = 0; }
    *total_us = 0; *busy_slot_us = 0; *n_prefill_iter = 0; *n_decode_iter = 0; *trace_hash = 0;
    if (trace_len) *trace_len = 0;
    for (int i = 0; i < N; i++)
        if (in_len[i] < 1 || out_len[i] < 1 || assign[i] < 0 || assign[i] >= cap) { *status = ST_BAD_SIM_INPUT; return; }

    /* the sorted queues I_j, stored one after the other in q[] */
    int *q = (int *)malloc((size_t)N * sizeof(int));
    int *qbeg = (int *)calloc((size_t)cap + 1, sizeof(int));
    int *head = (int *)malloc((size_t)cap * sizeof(int)), *th = (int *)malloc((size_t)cap * sizeof(int));
    int64_t *remain = (int64_t *)calloc((size_t)cap, sizeof(int64_t)), *tr_ = (int64_t *)malloc((size_t)cap * sizeof(int64_t));
    int32_t *run_req = (int32_t *)malloc((size_t)cap * sizeof(int32_t)), *run_rem = (int32_t *)malloc((size_t)cap * sizeof(int32_t));
    int *pick_client = (int *)malloc((size_t)cap * sizeof(int)), *pick_req = (int *)malloc((size_t)cap * sizeof(int));
    for (int i = 0; i < N; i++) qbeg[assign[i] + 1]++;
    for (int j = 0; j < cap; j++) qbeg[j + 1] += qbeg[j];
    for (int j = 0; j < cap; j++) head[j] = qbeg[j];
    for (int i = 0; i < N; i++) {                       /* insertion into I_j, longest first */
        int j = assign[i];
        int64_t len = (int64_t)in_len[i] + out_len[i];
        int pos = head[j]++;
        while (pos > qbeg[j] && (int64_t)in_len[q[pos - 1]] + out_len[q[pos - 1]] < len) { q[pos] = q[pos - 1]; pos--; }
        q[pos] = i;
        remain[j] += len;
    }
    for (int j = 0; j < cap; j++) { head[j] = qbeg[j]; run_req[j] = -1; run_rem[j] = 0; }

    int nR = 0, done = 0;
    int64_t t = 0, Cd = 0, busy = 0;
    int32_t npre = 0, ndec = 0;
    trace_t tr; memset(&tr, 0, sizeof tr);
    tr.hash = oracle_fnv1a64_init(); tr.buf = trace_buf; tr.cap = trace_capacity;

    while (done < N) {
        /* what the idle clients would take now, in client order (nothing is taken yet) */
        int nA = 0; int64_t P = 0;
        for (int j = 0; j < cap; j++) { th[j] = head[j]; tr_[j] = remain[j]; }
        for (int j = 0; j < cap; j++) {
            if (run_req[j] >= 0) continue;
            if (p->policy == 2 && nA >= 1) break;
            int src = -1;
            if (th[j] < qbeg[j + 1]) src = j;
            else {
                int64_t best = 0;
                for (int v = 0; v < cap; v++) if (tr_[v] > best) { best = tr_[v]; src = v; }
            }
            if (src < 0) continue;
            int req = q[th[src]];
            int64_t tok = in_len[req];
            if (p->max_prefill_tokens > 0 && P + tok > p->max_prefill_tokens && nA > 0) break;
            pick_client[nA] = j; pick_req[nA] = req;
            th[src]++; tr_[src] -= (int64_t)in_len[req] + out_len[req];
            P += tok; nA++;
            if (p->max_prefill_tokens > 0 && P > p->max_prefill_tokens) break;   /* oversized first pick: alone */
        }
        if (nA == 0 && nR == 0) break;       /* cannot happen while requests are left */
        int do_prefill;
        if (nA == 0) do_prefill = 0;
        else if (p->policy != 0) do_prefill = 1;
        else {
            int64_t Cp = p->a_prefill * P + p->c_prefill;
            if (nR == 0) do_prefill = 1;
            else if (Cp >= Cd) do_prefill = 0;
            else do_prefill = 1;
        }
        if (do_prefill) {
            int64_t dt = p->a_prefill * P + p->c_prefill;
            trace_other(&tr, 1, (uint32_t)nA, t, P);
            t += dt;
            for (int j = 0; j < cap; j++) { head[j] = th[j]; remain[j] = tr_[j]; }
            for (int k = 0; k < nA; k++) {
                int j = pick_client[k], req = pick_req[k];
                run_req[j] = req; run_rem[j] = out_len[req];
                if (served_by) served_by[req] = j;
                if (start_us) start_us[req] = t - dt;      /* start of the prefill iteration */
            }
            nR += nA;
            busy += (int64_t)nA * dt;
            Cd = 0;
            npre++;
        } else {
            int64_t D = nR;
            int64_t dt = p->b_decode * D + p->c_decode;
            trace_decode(&tr, t, D);
            t += dt;
            for (int j = 0; j < cap; j++) {
                if (run_req[j] < 0) continue;
                run_rem[j] -= 1;
                if (run_rem[j] == 0) { finish[run_req[j]] = t; run_req[j] = -1; done++; nR--; }
            }
            busy += D * dt;
            Cd += p->b_decode * D;
            ndec++;
        }
    }
    trace_flush(&tr);
    *total_us = t; *busy_slot_us = busy; *n_prefill_iter = npre; *n_decode_iter = ndec;
    *trace_hash = tr.hash;
    if (trace_len) *trace_len = tr.len;
    *status = done == N ? ST_OK : ST_BAD_SIM_INPUT;
    free(q); free(qbeg); free(head); free(th); free(remain); free(tr_); free(run_req); free(run_rem);
    free(pick_client); free(pick_req);
}

int oracle_online_iter_sim_assigned(const int32_t *in_len, const int32_t *out_len, const int32_t *assign,
                                    int S, int N, const oracle_sim_params *p, int64_t *finish_us,
                                    int64_t *total_us, int64_t *busy_slot_us, int32_t *n_prefill_iter,
                                    int32_t *n_decode_iter, uint64_t *trace_hash, int32_t *served_by,
                                    int64_t *start_us, void *trace_buf, int32_t *trace_len, int trace_scenarios,
                                    int trace_capacity, int32_t *status_out)
{
    if (!in_len || !out_len || !assign || !p || !finish_us || !total_us || !busy_slot_us ||
        !n_prefill_iter || !n_decode_iter || !trace_hash || !status_out) return -1;
    if (S <= 0 || N <= 0 || p->cap <= 0 || p->policy < 0 || p->policy > 2) return -1;
    if (p->a_prefill < 0 || p->b_decode < 0 || p->c_prefill < 0 || p->c_decode < 0) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int s = 0; s < S; s++) {
        int traced = trace_buf && s < trace_scenarios;
        sim_assigned_one(in_len + (size_t)s * N, out_len + (size_t)s * N, assign + (size_t)s * N, N, p,
                         finish_us + (size_t)s * N, total_us + s, busy_slot_us + s, n_prefill_iter + s,
                         n_decode_iter + s, trace_hash + s, served_by ? served_by + (size_t)s * N : 0,
                         start_us ? start_us + (size_t)s * N : 0,
                         traced ? (trace_rec *)trace_buf + (size_t)s * trace_capacity : 0,
                         traced ? trace_capacity : 0, (trace_len && s < trace_scenarios) ? trace_len + s : 0,
                         status_out + s);
    }
    return 0;
}

/* affine iteration-time model of the paper's experiment section, exposed for the worked-example pins */
int64_t oracle_prefill_time(const oracle_sim_params *p, int64_t tokens) { return p->a_prefill * tokens + p->c_prefill; }
int64_t oracle_decode_time(const oracle_sim_params *p, int64_t seqs) { return p->b_decode * seqs + p->c_decode; }
