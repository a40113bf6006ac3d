/*
 * libmmbp -- batched Minimizing Makespan Bin Packing (MMBP) local search, theoretical lower
 * bound and online iteration-scheduling simulator for gfx950 (MI355X).
 *
 * Vocabulary follows the paper's problem statement: requests i with N^p_i input and N^d_i
 * output tokens, clients / instances j (M of them), estimated completion cost T_i, per-client
 * load t_j, prefill / decode time per token T^p / T^d.
 *
 * Conventions for every entry point
 *   - plain C ABI; all array arguments are DEVICE pointers owned by the caller unless the
 *     comment says "host"; the library never frees or keeps them;
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is enqueued
 *     asynchronously on it; the library never synchronises the stream, so outputs are valid
 *     once the caller has synchronised;
 *   - return value: 0 = enqueued; negative = MMBP_E* (nothing was enqueued);
 *   - conditions only visible on the device are reported per scenario in `status_out`
 *     (MMBP_ST_*).  Scenarios are independent: a bad one does not affect the others.
 */
#ifndef MMBP_H
#define MMBP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* return codes */
#define MMBP_OK            0
#define MMBP_EINVAL       -1  /* null pointer, non-positive size, bad dtype, negative max_passes, unknown policy */
#define MMBP_EINFEASIBLE  -2  /* N > M * cap: no assignment satisfies the cardinality limit */
#define MMBP_EUNSUPPORTED -3  /* outside the supported range (N <= 2^20, M <= 256, sim cap <= 256,
                                 assigned simulator N <= 8192, max_passes <= MMBP_GRID_MAX_PASSES for a
                                 scenario that does not fit one workgroup's LDS) */
#define MMBP_EWORKSPACE   -4  /* workspace missing, smaller than mmbp_workspace_bytes(), or not 256-byte aligned */
#define MMBP_EHIP         -5  /* a HIP call or kernel launch failed; see mmbp_strerror() */

/* per-scenario status */
#define MMBP_ST_OK            0  /* converged: a full scan found no improving candidate */
#define MMBP_ST_TRUNCATED     1  /* max_passes reached before a scan proved local optimality */
#define MMBP_ST_BAD_ASSIGN    2  /* assign entry outside [0,M) or more than cap jobs on a client */
#define MMBP_ST_BAD_COST      3  /* negative cost, sum of costs >= 2^62, or (lower bound) a negative token count */
#define MMBP_ST_BAD_SIM_INPUT 4  /* arrival negative or decreasing, in_len < 1, out_len < 1 */
#define MMBP_ST_INTERNAL      5  /* a consistency check inside a kernel failed (a bug): the scenario's
                                    outputs are not valid */

/* cost element type */
#define MMBP_I32 0
#define MMBP_I64 1

#define MMBP_MAX_N (1 << 20)
#define MMBP_MAX_M 256
#define MMBP_GRID_MAX_PASSES 4096   /* candidates one call can apply on the multi-workgroup path */
#define MMBP_SIM_MAX_CAP 256
#define MMBP_SIM_ASSIGNED_MAX_N 8192

int mmbp_version(void);

/* Text for a return code; for MMBP_EHIP the text of the last failing HIP call of this thread.
 * The pointer is to static / thread-local storage. */
const char *mmbp_strerror(int code);

/*
 * Scratch for mmbp_local_search with these shapes (bytes of device memory; the base must be
 * 256-byte aligned).  0: every scenario is searched entirely out of the LDS of one workgroup.
 * Otherwise the call runs the multi-workgroup path, whose layout, per-row minima and task table
 * live in the workspace.  That path is REQUIRED when a scenario does not fit the LDS (larger N:
 * without the workspace the call returns MMBP_EWORKSPACE) and merely PREFERRED for a few large
 * scenarios that would leave most of the chip idle (at most 128 scenarios and a predicted factor
 * of two): there a call without workspace, or with one that is too small or misaligned, still
 * runs, on the one-workgroup path (as do mmbp_local_search_pruned and a call with max_passes above
 * 4096 for every scenario that fits).
 * Results do not depend on the path.
 */
size_t mmbp_workspace_bytes(int S, int N, int M);

/*
 * Measurement aid, no part of the method: runs the instruction mix of the local search's swap
 * evaluation (one 32-bit subtract per candidate, one three-way min and one three-way max per two
 * candidates) on registers only, so that a caller can time the vector-ALU issue rate the device
 * sustains and set the search's throughput against it.
 * out       device [blocks * 256] uint32 (receives one word per thread; its content means nothing)
 * blocks    workgroups of 256 threads, 1 .. 2^20;  trips: loop trips per thread, 1 .. 2^24
 * lane_ops  HOST pointer, nullable: receives the number of 32-bit lane operations the launch issues
 */
int mmbp_valu_probe(uint32_t *out, int blocks, int trips, uint64_t *lane_ops /* host */, void *stream);

/*
 * Theoretical lower bound, paper section "Offline requests scheduling & theoretical lower
 * bound": T^LB = t^p* + t^d*.
 *   t^d* (optimum of the MMBP model) is replaced by the largest of three relaxation bounds,
 *        ceil(sum_i T_i / M), max_i T_i, and T_(M) + T_(M+1) (costs in descending order, N > M);
 *   t^p* = tp_L * floor(sum_i prefill_tokens_i / ncap_L)  (the paper's floor form with the
 *        largest level L), added only when prefill_tokens != NULL and ncap_L > 0.
 * cost            [S,N] int32 or int64 per `dtype`, T_i >= 0
 * prefill_tokens  [S,N] int32 N^p_i >= 0, nullable (a negative entry, when the term is enabled, makes the
 *                 scenario MMBP_ST_BAD_COST)
 * lb_out          [S] int64
 * status_out      [S] int32: MMBP_ST_OK or MMBP_ST_BAD_COST (then lb_out = 0)
 */
int mmbp_lower_bound(const void *cost, int dtype, int S, int N, int M,
                     const int32_t *prefill_tokens, int64_t ncap_L, int64_t tp_L,
                     int64_t *lb_out, int32_t *status_out, void *stream);

/*
 * The same bound T^LB = t^p* + t^d* with stronger relaxations of t^d* and a level table for t^p*
 * (levels l of the paper's prefill-length constraints: a prefill stage of level l holds at most
 * N^cap_l tokens and takes T^p_l).
 *   L1 = ceil(sum_i T_i / M), L2 = max_i T_i as in mmbp_lower_bound;
 *   L3(k) = T_(kM+1) + T_(kM) + ... + T_(kM+1-k) (descending order): of the kM+1 largest requests
 *           some client holds k+1.  Evaluated for every k >= 1 with kM+1 <= min(N, MMBP_LB_RANK_LIMIT)
 *           and, if kmax > 0, k <= kmax; L3 = the largest of them (k = 1 is mmbp_lower_bound's term);
 *   Lcap  with per-client cardinality limits cap[j]: client j holds at least
 *           n_j = max(0, N - sum_{j' != j} cap[j']) requests, hence at least the n_j smallest costs;
 *           Lcap = sum of the max_j n_j smallest costs;
 *   t^p*  tp_form MMBP_TP_FLOOR_LARGEST: the paper's form T^p_L * floor(sum_i N^p_i / N^cap_L) on the
 *           level L of largest capacity (equal capacities: the smaller time);
 *         tp_form MMBP_TP_COVER: min_l ceil(sum_i N^p_i * T^p_l / N^cap_l), a bound for every table
 *           (stages that cover all tokens cannot beat the most efficient level's time per token).
 *   lb = max(L1, L2, L3, Lcap) + t^p*.
 * cost            [S,N] int32 or int64 per `dtype`, T_i >= 0
 * cap             HOST [M] int32, nullable (no limits); sum cap[j] < N returns MMBP_EINFEASIBLE
 * prefill_tokens  [S,N] int32 N^p_i >= 0, nullable; the t^p* term needs it and n_levels > 0
 * ncap, tp        HOST [n_levels] int64, 1 <= ncap[l] < 2^31, 0 <= tp[l] < 2^31; n_levels <= MMBP_LB_MAX_LEVELS
 * lb_out          [S] int64
 * parts_out       [S,6] int64, nullable: L1, L2, L3, the smallest k that attains L3 (0: none), Lcap, t^p*
 * status_out      [S] int32: MMBP_ST_OK, or MMBP_ST_BAD_COST (negative cost or token count, sum of costs
 *                 or t^p* not below 2^62): then lb_out and parts_out of the scenario are 0
 */
#define MMBP_TP_FLOOR_LARGEST 0
#define MMBP_TP_COVER         1
#define MMBP_LB_RANK_LIMIT    16384
#define MMBP_LB_MAX_LEVELS    16
int mmbp_lower_bound_ex(const void *cost, int dtype, int S, int N, int M, const int32_t *cap /* host */, int kmax,
                        const int32_t *prefill_tokens, int n_levels, const int64_t *ncap /* host */,
                        const int64_t *tp /* host */, int tp_form, int64_t *lb_out, int64_t *parts_out,
                        int32_t *status_out, void *stream);

/*
 * A start for the local search: the longest-processing-time rule on the MMBP model (same section;
 * objective min max_j t_j) with at most `cap` requests per client.  The requests are taken by
 * decreasing T_i (equal costs: lower index first) and each goes to the client with the smallest load
 * among those that still have room (equal loads: lower client index).  With cap >= N the makespan is
 * at most (4/3 - 1/(3M)) times the optimum of the model.
 * cost        [S,N] int32 / int64 per `dtype`, T_i >= 0;  N <= MMBP_LPT_MAX_N
 * assign_out  [S,N] int32: the client of every request (a feasible start for mmbp_local_search)
 * load_out    [S,M] int64 t_j of that assignment
 * order_out   [S,N] int32: the request indices in the order they were taken (required: the kernel
 *             also uses it to hand the order from its sorting phase to its assignment phase)
 * status_out  [S] int32: MMBP_ST_OK, or MMBP_ST_BAD_COST (then assign_out and order_out are -1, loads 0)
 * Returns MMBP_EINFEASIBLE when N > M * cap.
 */
#define MMBP_LPT_MAX_N 16384
int mmbp_lpt_start(const void *cost, int dtype, int S, int N, int M, int cap, int32_t *assign_out,
                   int64_t *load_out, int32_t *order_out, int32_t *status_out, void *stream);

/*
 * Best-improvement local search on the MMBP model (same section: min max_j t_j, every request
 * on exactly one client, t_j = sum of the T_i assigned to j), with at most `cap` requests per
 * client.  Each pass evaluates the makespan that EVERY candidate would give,
 *   move  (i -> b),  b != assign[i], feasible iff count(b) + 1 <= cap,   id = i*M + b
 *   swap  (i <-> k), i < k, assign[i] != assign[k],                      id = N*M + i*N + k
 * takes the candidate with the smallest (makespan, id) and applies it if it lowers the
 * makespan; otherwise the search stops (MMBP_ST_OK).  It also stops after max_passes applied
 * candidates (MMBP_ST_TRUNCATED; max_passes = 0 only reports the loads of the start).  `assign`
 * is in/out, so a truncated search is resumed by calling again: k passes followed by k more give
 * exactly what 2k passes give.  A scenario too large for one workgroup's LDS (mmbp_workspace_bytes)
 * is searched with a fixed number of launches per pass, enqueued up front; for such shapes
 * max_passes above MMBP_GRID_MAX_PASSES returns MMBP_EUNSUPPORTED (nothing is enqueued) and the
 * caller resumes in calls of at most that many passes.
 * cost         [S,N] int32 / int64 per `dtype`
 * assign       [S,N] int32, in: feasible start, out: result (untouched for bad scenarios)
 * load_out     [S,M] int64 t_j of the result;  makespan_out [S] int64;  passes_out [S] int32
 * evals_out    [S] uint64, nullable: candidates enumerated over all scans, counting capacity-
 *              infeasible moves, not counting b == assign[i] nor same-client pairs
 * applied_log  [S,max_passes] uint64, nullable: id applied in each pass (rest untouched)
 * status_out   [S] int32.  For MMBP_ST_BAD_*: load/makespan/passes/evals are 0.
 * workspace    device scratch of at least mmbp_workspace_bytes(S,N,M) bytes (may be NULL if that is 0, or
 *              where the multi-workgroup path is only preferred, see mmbp_workspace_bytes)
 */
int mmbp_local_search(const void *cost, int dtype, int S, int N, int M, int cap, int max_passes,
                      int32_t *assign, int64_t *load_out, int64_t *makespan_out,
                      int32_t *passes_out, uint64_t *evals_out, uint64_t *applied_log,
                      int32_t *status_out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * The same search with a pruned scan.  The objective of the MMBP model (same section) is
 * max_j t_j, so a candidate lowers it only if it takes load off the client that attains it: each
 * pass evaluates only the moves off that client and the swaps with it, and stops when none of
 * them improves.  Assignments, loads, makespans, pass counts, applied_log and status are identical
 * to mmbp_local_search on every input.  evals_out reports the candidates a full scan would have
 * enumerated (the same numbers mmbp_local_search reports), not the smaller number evaluated here.
 * Arguments, workspace and error behaviour as for mmbp_local_search; a scenario that fits one
 * workgroup's LDS is always searched there (each client's costs are kept sorted and the best partner of
 * a request is found by binary search, or against all of them where they are few), and more shapes fit
 * than for the full scan, which needs tables
 * for its tiles: for those the workspace may be NULL although mmbp_workspace_bytes() is not 0.
 */
int mmbp_local_search_pruned(const void *cost, int dtype, int S, int N, int M, int cap, int max_passes,
                             int32_t *assign, int64_t *load_out, int64_t *makespan_out,
                             int32_t *passes_out, uint64_t *evals_out, uint64_t *applied_log,
                             int32_t *status_out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * mmbp_local_search for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results,
 * status codes and path selection as mmbp_local_search, without the workspace pair: where that call
 * would use a workspace, this one uses a scratch array that is part of the library's device code
 * (MMBP_STATIC_SCRATCH_BYTES per GPU, held from the moment the library is loaded on that GPU until
 * the process ends).  The call allocates and frees nothing, on the host side of the GPU or through
 * any library; its first call on a device looks the array's device address up once (not an
 * allocation; make that first call outside a graph capture).
 *   - mmbp_workspace_bytes(S,N,M) above MMBP_STATIC_SCRATCH_BYTES: MMBP_EWORKSPACE (nothing is
 *     enqueued) when the shape needs the multi-workgroup path; where that path is only preferred the
 *     one-workgroup path runs instead.
 *   - All calls on one GPU share that GPU's array (it keeps the last call's contents; the kernels
 *     initialise what they read).  Two calls that overlap in time on one GPU (different streams, or
 *     different host threads without stream order between them) race on it: keep them in stream order.
 */
#define MMBP_STATIC_SCRATCH_BYTES (16u << 20)
int mmbp_local_search_static(const void *cost, int dtype, int S, int N, int M, int cap, int max_passes,
                             int32_t *assign, int64_t *load_out, int64_t *makespan_out,
                             int32_t *passes_out, uint64_t *evals_out, uint64_t *applied_log,
                             int32_t *status_out, void *stream);

/* Iteration-scheduling policy of the simulator.
 * MMBP_POLICY_RULE: the paper's rule (section "Online requests and iteration scheduling"):
 *     C_p >= C_d keeps decoding, otherwise the prefill is dispatched.
 * MMBP_POLICY_PREFILL_FIRST: the baseline the paper measures against (FCFS, prefill first, see its
 *     introduction and section "Experiment settings and baseline"): whenever an arrived request
 *     finds a free slot, the prefill of the admissible requests is dispatched at the next boundary.
 * MMBP_POLICY_PREFILL_FIRST_SINGLE: the same, one request per prefill iteration (the paper notes
 *     that the baseline does not process several requests in one prefill stage). */
#define MMBP_POLICY_RULE                 0
#define MMBP_POLICY_PREFILL_FIRST        1
#define MMBP_POLICY_PREFILL_FIRST_SINGLE 2

/* Parameters of the iteration simulator (HOST struct).  Times in integer microseconds.
 * Affine time model of the paper's section "Experiment settings and baseline":
 * a prefill iteration over P tokens takes a_prefill*P + c_prefill, a decode iteration over D
 * running requests takes b_decode*D + c_decode. */
typedef struct mmbp_sim_params {
    int32_t cap;                /* batch size |J|: requests processed simultaneously, 1..256 */
    int32_t policy;             /* MMBP_POLICY_* */
    int64_t a_prefill;          /* T^p per token */
    int64_t b_decode;           /* T^d per token (one token per running request per round) */
    int64_t c_prefill;          /* fixed prefill overhead */
    int64_t c_decode;           /* fixed decode overhead */
    int64_t max_prefill_tokens; /* token capacity of a prefill iteration; <= 0: unlimited */
} mmbp_sim_params;

/* One canonical trace record (24 bytes, little endian). kind 0 = DECODE run (count iterations
 * with x = D running requests each), 1 = PREFILL (count = requests admitted, x = tokens P),
 * 2 = IDLE jump to the next arrival (count 1, x 0). */
typedef struct mmbp_trace_rec {
    uint32_t kind, count;
    int64_t t_start, x;
} mmbp_trace_rec;

/*
 * Iteration-level simulation of one node under PD competition (an iteration is either a
 * prefill or a decode), paper section "Online requests and iteration scheduling": at every
 * iteration boundary the admissible requests (FCFS prefix of the arrived ones that fits the
 * free slots and the token capacity) define the prefill cost C_p = a_prefill*P + c_prefill;
 * the waited decode time C_d is b_decode times the tokens decoded since the last prefill.
 * C_p >= C_d keeps decoding, otherwise the prefill is dispatched (params->policy selects the
 * baseline policies instead); with nothing running the prefill is forced; with nothing running
 * and nothing arrived time jumps to the next arrival.
 * arrival_us [S,N] int64 nondecreasing along N; in_len, out_len [S,N] int32 >= 1
 * finish_us  [S,N] int64;  total_us, busy_slot_us [S] int64;  n_prefill_iter, n_decode_iter [S]
 * trace_hash [S] uint64: FNV-1a (64 bit) over the canonical records
 * trace_buf  nullable, [trace_scenarios, trace_capacity] mmbp_trace_rec for the first
 *            trace_scenarios scenarios; trace_len [trace_scenarios] int32 = records produced
 *            (may exceed trace_capacity; only the first trace_capacity are stored)
 * status_out [S]: MMBP_ST_OK or MMBP_ST_BAD_SIM_INPUT (then every output of the scenario is 0)
 */
int online_iter_sim(const int64_t *arrival_us, const int32_t *in_len, const int32_t *out_len,
                    int S, int N, const mmbp_sim_params *params /* host */,
                    int64_t *finish_us, int64_t *total_us, int64_t *busy_slot_us,
                    int32_t *n_prefill_iter, int32_t *n_decode_iter, uint64_t *trace_hash,
                    mmbp_trace_rec *trace_buf, int32_t *trace_len, int trace_scenarios,
                    int trace_capacity, int32_t *status_out, void *stream);

/*
 * The iteration simulator fed by an offline assignment (for example the result of
 * mmbp_local_search with M = params->cap clients): request scheduling by the sorting and online
 * preemptive method of the paper's section "Online requests and iteration scheduling".
 *   I_j = the requests with assign == j, sorted by in_len + out_len, longest first (equal lengths:
 *   lower index first); remain_token(j) = sum of in_len + out_len over what is left in I_j.  At an
 *   iteration boundary the clients are visited in index order: an idle client takes the head of
 *   its own I_j if there is one, otherwise the head of the I_v with the largest positive
 *   remain_token (lowest v among equals).  The requests picked form the prefill that could be
 *   dispatched (cut by max_prefill_tokens like the FCFS prefix; the first pick always fits); the
 *   decision between prefill and decode, the time model, the trace and all other outputs are those
 *   of online_iter_sim, and picks are only taken when the prefill is dispatched.  All requests are
 *   known at t = 0 (the method works on the offline request set): there are no arrival times.
 * in_len, out_len [S,N] int32 >= 1;  assign [S,N] int32 in [0, params->cap)
 * served_by  nullable, [S,N] int32: the client that ran the request (differs from assign when stolen)
 * start_us   nullable, [S,N] int64: start of the prefill iteration that admitted the request
 * status_out [S]: MMBP_ST_OK or MMBP_ST_BAD_SIM_INPUT (then every output of the scenario is 0 and
 *            served_by is -1)
 * N <= MMBP_SIM_ASSIGNED_MAX_N (the queues of a scenario are kept in LDS).
 */
int online_iter_sim_assigned(const int32_t *in_len, const int32_t *out_len, const int32_t *assign, int S, int N,
                             const mmbp_sim_params *params /* host */, int64_t *finish_us, int64_t *total_us,
                             int64_t *busy_slot_us, int32_t *n_prefill_iter, int32_t *n_decode_iter,
                             uint64_t *trace_hash, int32_t *served_by, int64_t *start_us,
                             mmbp_trace_rec *trace_buf, int32_t *trace_len, int trace_scenarios,
                             int trace_capacity, int32_t *status_out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MMBP_H */
