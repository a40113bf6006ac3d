// C-ABI boundary of libmmbp: argument validation, path selection, kernel launches on the caller's
// stream.  No allocation, no synchronisation.
#include <climits>
#include <cstdio>
#include <cstring>
#include <mutex>
#include "mmbp_dev.hpp"

namespace {
thread_local char g_hip_err[256] = "no HIP error recorded";

int fail_hip(hipError_t e, const char *where)
{
    snprintf(g_hip_err, sizeof g_hip_err, "%s: %s", where, hipGetErrorString(e));
    return MMBP_EHIP;
}
}  // namespace

// ---- the entry point that allocates nothing ----
// Scratch of the multi-workgroup path for callers that cannot bring a workspace: one array per GPU
// (each device that loads this code object holds its own copy at its own address until the process
// ends).  In host code the array's name is only a handle; the device address is looked up once per
// device and that pointer is what the kernels get.
constexpr size_t kStaticScratchBytes = MMBP_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

// device address of `scratch` on the current device (looked up on the first call per device)
int static_scratch(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e, "mmbp_local_search_static(hipGetDevice)");
    if (dev < 0 || dev >= kMaxDevices) return MMBP_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return fail_hip(e, "mmbp_local_search_static(hipGetSymbolAddress)");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return MMBP_OK;
}
}  // namespace

extern "C" {

int mmbp_version(void) { return 100; }

const char *mmbp_strerror(int code)
{
    switch (code) {
    case MMBP_OK: return "ok";
    case MMBP_EINVAL: return "invalid argument (null pointer, non-positive size, bad dtype, negative max_passes or unknown policy)";
    case MMBP_EINFEASIBLE: return "infeasible: N > M * cap";
    case MMBP_EUNSUPPORTED: return "unsupported size (N <= 2^20, M <= 256, simulator cap <= 256, assigned simulator N <= 8192, "
                                   "max_passes <= 4096 per call for scenarios that need the multi-workgroup path)";
    case MMBP_EWORKSPACE: return "workspace missing, too small or not 256-byte aligned (see mmbp_workspace_bytes), or the "
                                 "shape needs more scratch than mmbp_local_search_static holds (MMBP_STATIC_SCRATCH_BYTES)";
    case MMBP_EHIP: return g_hip_err;
    default: return "unknown error code";
    }
}

// A few large scenarios leave most of the chip idle on the one-workgroup-per-scenario path, where a
// pass of a scenario costs about 4 us + 14 ns per 1000 swap candidates on its CU; the multi-workgroup
// path costs about 19 us per pass plus 0.3 us + 0.11 ns per 1000 candidates per scenario (both
// measured on MI355X).  It is preferred where this predicts at least a factor of two.
static bool prefer_multi_workgroup(int S, int N, int M)
{
    if (S > 128) return false;
    const double pairs = 0.5 * (double)N * (double)N * (1.0 - 1.0 / (double)M);
    const double one_wg = 4.0 + 14e-6 * pairs;
    const double multi_wg = 19.0 + (double)S * (0.3 + 0.11e-6 * pairs);
    return 2.0 * multi_wg < one_wg;
}

size_t mmbp_workspace_bytes(int S, int N, int M)
{
    if (S <= 0 || N <= 0 || M <= 0 || N > MMBP_MAX_N || M > MMBP_MAX_M) return 0;
    if (mmbp::ls_lds_fits(N, M, false) && !prefer_multi_workgroup(S, N, M)) return 0;
    return mmbp::ls_grid_workspace_bytes(S, N, M);
}

int mmbp_valu_probe(uint32_t *out, int blocks, int trips, uint64_t *lane_ops, void *stream)
{
    if (!out || blocks <= 0 || trips <= 0) return MMBP_EINVAL;
    if (blocks > (1 << 20) || trips > (1 << 24)) return MMBP_EUNSUPPORTED;
    if (lane_ops) *lane_ops = (uint64_t)blocks * 256ull * (uint64_t)trips * (uint64_t)mmbp::valu_probe_ops_per_trip();
    hipError_t e = mmbp::launch_valu_probe(out, blocks, trips, (hipStream_t)stream);
    return e == hipSuccess ? MMBP_OK : fail_hip(e, "mmbp_valu_probe");
}

int mmbp_lower_bound(const void *cost, int dtype, int S, int N, int M, const int32_t *prefill_tokens,
                     int64_t ncap_L, int64_t tp_L, int64_t *lb_out, int32_t *status_out, void *stream)
{
    if (!cost || !lb_out || !status_out) return MMBP_EINVAL;
    if (S <= 0 || N <= 0 || M <= 0) return MMBP_EINVAL;
    if (dtype != MMBP_I32 && dtype != MMBP_I64) return MMBP_EINVAL;
    if (ncap_L < 0 || tp_L < 0) return MMBP_EINVAL;
    if (N > MMBP_MAX_N || M > MMBP_MAX_M) return MMBP_EUNSUPPORTED;
    hipError_t e = mmbp::launch_lower_bound(cost, dtype, S, N, M, prefill_tokens, ncap_L, tp_L, lb_out, status_out,
                                            (hipStream_t)stream);
    return e == hipSuccess ? MMBP_OK : fail_hip(e, "mmbp_lower_bound");
}

int mmbp_lower_bound_ex(const void *cost, int dtype, int S, int N, int M, const int32_t *cap, int kmax,
                        const int32_t *prefill_tokens, int n_levels, const int64_t *ncap, const int64_t *tp, int tp_form,
                        int64_t *lb_out, int64_t *parts_out, int32_t *status_out, void *stream)
{
    if (!cost || !lb_out || !status_out) return MMBP_EINVAL;
    if (S <= 0 || N <= 0 || M <= 0) return MMBP_EINVAL;
    if (dtype != MMBP_I32 && dtype != MMBP_I64) return MMBP_EINVAL;
    if (n_levels < 0 || (n_levels > 0 && (!ncap || !tp))) return MMBP_EINVAL;
    if (tp_form != MMBP_TP_FLOOR_LARGEST && tp_form != MMBP_TP_COVER) return MMBP_EINVAL;
    if (N > MMBP_MAX_N || M > MMBP_MAX_M || n_levels > MMBP_LB_MAX_LEVELS) return MMBP_EUNSUPPORTED;
    for (int l = 0; l < n_levels; l++)
        if (ncap[l] < 1 || ncap[l] > INT32_MAX || tp[l] < 0 || tp[l] > INT32_MAX) return MMBP_EINVAL;
    int nstar = 0;                                       // the most requests the limits force onto one client
    if (cap) {
        int64_t capsum = 0;
        for (int j = 0; j < M; j++) {
            if (cap[j] < 0) return MMBP_EINVAL;
            capsum += cap[j];
        }
        if (capsum < N) return MMBP_EINFEASIBLE;
        for (int j = 0; j < M; j++) {
            const int64_t nj = (int64_t)N - (capsum - cap[j]);
            if (nj > nstar) nstar = (int)nj;
        }
    }
    int K = (N - 1) / M;                                 // terms L3(k): k*M + 1 <= N, within the rank limit and the caller's
    if (K > (MMBP_LB_RANK_LIMIT - 1) / M) K = (MMBP_LB_RANK_LIMIT - 1) / M;
    if (kmax > 0 && K > kmax) K = kmax;
    hipError_t e = mmbp::launch_lower_bound_ex(cost, dtype, S, N, M, K, nstar, prefill_tokens, n_levels, ncap, tp, tp_form,
                                               lb_out, parts_out, status_out, (hipStream_t)stream);
    return e == hipSuccess ? MMBP_OK : fail_hip(e, "mmbp_lower_bound_ex");
}

int mmbp_lpt_start(const void *cost, int dtype, int S, int N, int M, int cap, int32_t *assign_out, int64_t *load_out,
                   int32_t *order_out, int32_t *status_out, void *stream)
{
    if (!cost || !assign_out || !load_out || !order_out || !status_out) return MMBP_EINVAL;
    if (S <= 0 || N <= 0 || M <= 0 || cap <= 0) return MMBP_EINVAL;
    if (dtype != MMBP_I32 && dtype != MMBP_I64) return MMBP_EINVAL;
    if (N > MMBP_LPT_MAX_N || M > MMBP_MAX_M) return MMBP_EUNSUPPORTED;
    if ((int64_t)N > (int64_t)M * (int64_t)cap) return MMBP_EINFEASIBLE;
    hipError_t e = mmbp::launch_lpt_start(cost, dtype, S, N, M, cap, assign_out, load_out, order_out, status_out,
                                          (hipStream_t)stream);
    return e == hipSuccess ? MMBP_OK : fail_hip(e, "mmbp_lpt_start");
}

static int local_search_impl(int prune, const void *cost, int dtype, int S, int N, int M, int cap, int max_passes, int32_t *assign,
                      int64_t *load_out, int64_t *makespan_out, int32_t *passes_out, uint64_t *evals_out,
                      uint64_t *applied_log, int32_t *status_out, void *workspace, size_t workspace_bytes,
                      void *stream)
{
    if (!cost || !assign || !load_out || !makespan_out || !passes_out || !status_out) return MMBP_EINVAL;
    if (S <= 0 || N <= 0 || M <= 0 || cap <= 0 || max_passes < 0) return MMBP_EINVAL;
    if (dtype != MMBP_I32 && dtype != MMBP_I64) return MMBP_EINVAL;
    if (N > MMBP_MAX_N || M > MMBP_MAX_M) return MMBP_EUNSUPPORTED;
    if ((int64_t)N > (int64_t)M * (int64_t)cap) return MMBP_EINFEASIBLE;
    const size_t need = mmbp_workspace_bytes(S, N, M);
    const bool ws_ok = need > 0 && workspace && workspace_bytes >= need && ((uintptr_t)workspace & 255u) == 0;
    const bool fits = mmbp::ls_lds_fits(N, M, prune != 0);
    if (!fits && !ws_ok) return MMBP_EWORKSPACE;
    // The multi-workgroup path enqueues its launches pass by pass and cannot see convergence from the
    // host: a call applies at most MMBP_GRID_MAX_PASSES candidates.  A larger limit on a shape that
    // needs this path is refused rather than silently cut (the caller resumes with further calls).
    if (!fits && max_passes > MMBP_GRID_MAX_PASSES) return MMBP_EUNSUPPORTED;
    // One workgroup per scenario: the fallback when the optional workspace is not given, and always
    // for the pruned scan of a scenario that fits (its pass is about as short as three launches),
    // and for a pass limit the multi-workgroup path cannot honour in one call.
    const bool one_wg = fits && (!ws_ok || prune != 0 || max_passes > mmbp::ls_grid_pass_limit());
    hipStream_t st = (hipStream_t)stream;

    // The first path writes a status for every scenario: final where it can search the scenario
    // exactly, pending otherwise; the 64-bit kernel then takes the pending ones.
    hipError_t e;
    if (one_wg) {
        e = mmbp::launch_ls_lds(cost, dtype, S, N, M, cap, max_passes, prune, assign, load_out, makespan_out, passes_out,
                                evals_out, applied_log, status_out, st);
        if (e != hipSuccess) return fail_hip(e, "mmbp_local_search(lds)");
    } else {
        e = mmbp::launch_ls_grid(cost, dtype, S, N, M, cap, max_passes, prune, assign, load_out, makespan_out, passes_out,
                                 evals_out, applied_log, status_out, workspace, st);
        if (e != hipSuccess) return fail_hip(e, "mmbp_local_search(grid)");
    }
    e = mmbp::launch_ls_generic(cost, dtype, S, N, M, cap, max_passes, assign, load_out, makespan_out, passes_out,
                                evals_out, applied_log, status_out, st);
    return e == hipSuccess ? MMBP_OK : fail_hip(e, "mmbp_local_search(generic)");
}

int mmbp_local_search(const void *cost, int dtype, int S, int N, int M, int cap, int max_passes, int32_t *assign,
                      int64_t *load_out, int64_t *makespan_out, int32_t *passes_out, uint64_t *evals_out,
                      uint64_t *applied_log, int32_t *status_out, void *workspace, size_t workspace_bytes,
                      void *stream)
{
    return local_search_impl(0, cost, dtype, S, N, M, cap, max_passes, assign, load_out, makespan_out, passes_out,
                             evals_out, applied_log, status_out, workspace, workspace_bytes, stream);
}

int mmbp_local_search_pruned(const void *cost, int dtype, int S, int N, int M, int cap, int max_passes,
                             int32_t *assign, int64_t *load_out, int64_t *makespan_out, int32_t *passes_out,
                             uint64_t *evals_out, uint64_t *applied_log, int32_t *status_out, void *workspace,
                             size_t workspace_bytes, void *stream)
{
    return local_search_impl(1, cost, dtype, S, N, M, cap, max_passes, assign, load_out, makespan_out, passes_out,
                             evals_out, applied_log, status_out, workspace, workspace_bytes, stream);
}

// ---- the entry point that allocates nothing (its scratch is declared above) ----
int mmbp_local_search_static(const void *cost, int dtype, int S, int N, int M, int cap, int max_passes, int32_t *assign,
                             int64_t *load_out, int64_t *makespan_out, int32_t *passes_out, uint64_t *evals_out,
                             uint64_t *applied_log, int32_t *status_out, void *stream)
{
    // argument errors first, exactly as mmbp_local_search reports them
    if (!cost || !assign || !load_out || !makespan_out || !passes_out || !status_out) return MMBP_EINVAL;
    if (S <= 0 || N <= 0 || M <= 0 || cap <= 0 || max_passes < 0) return MMBP_EINVAL;
    if (dtype != MMBP_I32 && dtype != MMBP_I64) return MMBP_EINVAL;
    if (N > MMBP_MAX_N || M > MMBP_MAX_M) return MMBP_EUNSUPPORTED;
    if ((int64_t)N > (int64_t)M * (int64_t)cap) return MMBP_EINFEASIBLE;
    const size_t need = mmbp_workspace_bytes(S, N, M);
    void *ws = nullptr;
    if (need > kStaticScratchBytes) {
        // where the multi-workgroup path is only preferred the one-workgroup path still runs
        if (!mmbp::ls_lds_fits(N, M, false)) return MMBP_EWORKSPACE;
    } else if (need > 0) {
        const int rc = static_scratch(&ws);
        if (rc != MMBP_OK) return rc;
    }
    return local_search_impl(0, cost, dtype, S, N, M, cap, max_passes, assign, load_out, makespan_out, passes_out,
                             evals_out, applied_log, status_out, ws, ws ? kStaticScratchBytes : 0, stream);
}

int online_iter_sim(const int64_t *arrival_us, const int32_t *in_len, const int32_t *out_len, int S, int N,
                    const mmbp_sim_params *params, int64_t *finish_us, int64_t *total_us, int64_t *busy_slot_us,
                    int32_t *n_prefill_iter, int32_t *n_decode_iter, uint64_t *trace_hash,
                    mmbp_trace_rec *trace_buf, int32_t *trace_len, int trace_scenarios, int trace_capacity,
                    int32_t *status_out, void *stream)
{
    if (!arrival_us || !in_len || !out_len || !params || !finish_us || !total_us || !busy_slot_us ||
        !n_prefill_iter || !n_decode_iter || !trace_hash || !status_out)
        return MMBP_EINVAL;
    if (S <= 0 || N <= 0 || params->cap <= 0) return MMBP_EINVAL;
    if (params->policy < MMBP_POLICY_RULE || params->policy > MMBP_POLICY_PREFILL_FIRST_SINGLE) return MMBP_EINVAL;
    if (params->a_prefill < 0 || params->b_decode < 0 || params->c_prefill < 0 || params->c_decode < 0)
        return MMBP_EINVAL;
    if (trace_buf && (trace_scenarios < 0 || trace_capacity < 0 || !trace_len)) return MMBP_EINVAL;
    if (params->cap > MMBP_SIM_MAX_CAP || N > MMBP_MAX_N) return MMBP_EUNSUPPORTED;
    if (!trace_buf) { trace_scenarios = 0; trace_capacity = 0; }
    hipError_t e = mmbp::launch_online_sim(arrival_us, in_len, out_len, S, N, *params, finish_us, total_us,
                                           busy_slot_us, n_prefill_iter, n_decode_iter, trace_hash, trace_buf,
                                           trace_buf ? trace_len : nullptr, trace_scenarios, trace_capacity,
                                           status_out, (hipStream_t)stream);
    return e == hipSuccess ? MMBP_OK : fail_hip(e, "online_iter_sim");
}

int online_iter_sim_assigned(const int32_t *in_len, const int32_t *out_len, const int32_t *assign, int S, int N,
                             const mmbp_sim_params *params, int64_t *finish_us, int64_t *total_us,
                             int64_t *busy_slot_us, int32_t *n_prefill_iter, int32_t *n_decode_iter,
                             uint64_t *trace_hash, int32_t *served_by, int64_t *start_us, mmbp_trace_rec *trace_buf,
                             int32_t *trace_len, int trace_scenarios, int trace_capacity, int32_t *status_out,
                             void *stream)
{
    if (!in_len || !out_len || !assign || !params || !finish_us || !total_us || !busy_slot_us || !n_prefill_iter ||
        !n_decode_iter || !trace_hash || !status_out)
        return MMBP_EINVAL;
    if (S <= 0 || N <= 0 || params->cap <= 0) return MMBP_EINVAL;
    if (params->policy < MMBP_POLICY_RULE || params->policy > MMBP_POLICY_PREFILL_FIRST_SINGLE) return MMBP_EINVAL;
    if (params->a_prefill < 0 || params->b_decode < 0 || params->c_prefill < 0 || params->c_decode < 0)
        return MMBP_EINVAL;
    if (trace_buf && (trace_scenarios < 0 || trace_capacity < 0 || !trace_len)) return MMBP_EINVAL;
    if (params->cap > MMBP_SIM_MAX_CAP || N > MMBP_SIM_ASSIGNED_MAX_N) return MMBP_EUNSUPPORTED;
    if (!trace_buf) { trace_scenarios = 0; trace_capacity = 0; }
    hipError_t e = mmbp::launch_online_sim_assigned(in_len, out_len, assign, S, N, *params, finish_us, total_us,
                                                    busy_slot_us, n_prefill_iter, n_decode_iter, trace_hash, served_by,
                                                    start_us, trace_buf, trace_buf ? trace_len : nullptr,
                                                    trace_scenarios, trace_capacity, status_out, (hipStream_t)stream);
    return e == hipSuccess ? MMBP_OK : fail_hip(e, "online_iter_sim_assigned");
}

}  // extern "C"
