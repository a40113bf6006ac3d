// Internal declarations shared by the HIP translation units of libmmbp (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/mmbp.h"

namespace mmbp {

constexpr int kWave = 64;
constexpr int32_t kPending = -1;          // status_out value while no path has taken the scenario
constexpr int64_t kCostSumLimit = (int64_t)1 << 62;

// ---- host-side launchers, one per translation unit (all enqueue on `st`, return hipError_t) ----
hipError_t launch_ls_generic(const void *cost, int dtype, int S, int N, int M, int cap, int max_passes,
                             int32_t *assign, int64_t *load_out, int64_t *makespan_out, int32_t *passes_out,
                             uint64_t *evals_out, uint64_t *applied_log, int32_t *status_out, hipStream_t st);

// LDS-resident path: true if shapes fit (N + 64*M padded positions in one workgroup's LDS; the pruned
// scan needs no tile tables, so more shapes fit it).
bool ls_lds_fits(int N, int M, bool prune);
hipError_t launch_ls_lds(const void *cost, int dtype, int S, int N, int M, int cap, int max_passes, int prune,
                         int32_t *assign, int64_t *load_out, int64_t *makespan_out, int32_t *passes_out,
                         uint64_t *evals_out, uint64_t *applied_log, int32_t *status_out, hipStream_t st);

// multi-workgroup path (large N): state in the caller's workspace
size_t ls_grid_workspace_bytes(int S, int N, int M);
int ls_grid_pass_limit();     // passes one call of the multi-workgroup path can apply (it then reports TRUNCATED)
hipError_t launch_ls_grid(const void *cost, int dtype, int S, int N, int M, int cap, int max_passes, int prune,
                          int32_t *assign, int64_t *load_out, int64_t *makespan_out, int32_t *passes_out,
                          uint64_t *evals_out, uint64_t *applied_log, int32_t *status_out, void *workspace,
                          hipStream_t st);

hipError_t launch_lower_bound(const void *cost, int dtype, int S, int N, int M, const int32_t *prefill_tokens,
                              int64_t ncap_L, int64_t tp_L, int64_t *lb_out, int32_t *status_out, hipStream_t st);

hipError_t launch_lower_bound_ex(const void *cost, int dtype, int S, int N, int M, int K, int nstar,
                                 const int32_t *prefill_tokens, int n_levels, const int64_t *ncap, const int64_t *tp,
                                 int tp_form, int64_t *lb_out, int64_t *parts_out, int32_t *status_out, hipStream_t st);

hipError_t launch_lpt_start(const void *cost, int dtype, int S, int N, int M, int cap, int32_t *assign_out,
                            int64_t *load_out, int32_t *order_out, int32_t *status_out, hipStream_t st);

hipError_t launch_online_sim(const int64_t *arrival_us, const int32_t *in_len, const int32_t *out_len, int S, int N,
                             const mmbp_sim_params &p, int64_t *finish_us, int64_t *total_us, int64_t *busy_slot_us,
                             int32_t *n_prefill_iter, int32_t *n_decode_iter, uint64_t *trace_hash,
                             mmbp_trace_rec *trace_buf, int32_t *trace_len, int trace_scenarios, int trace_capacity,
                             int32_t *status_out, hipStream_t st);
size_t sim_assigned_lds_bytes(int N);
hipError_t launch_online_sim_assigned(const int32_t *in_len, const int32_t *out_len, const int32_t *assign, int S, int N,
                                      const mmbp_sim_params &p, int64_t *finish_us, int64_t *total_us,
                                      int64_t *busy_slot_us, int32_t *n_prefill_iter, int32_t *n_decode_iter,
                                      uint64_t *trace_hash, int32_t *served_by, int64_t *start_us,
                                      mmbp_trace_rec *trace_buf, int32_t *trace_len, int trace_scenarios,
                                      int trace_capacity, int32_t *status_out, hipStream_t st);

// calibration probe of the vector-ALU issue rate (measurement aid, see valu_probe.hip)
int valu_probe_ops_per_trip();
hipError_t launch_valu_probe(uint32_t *out, int blocks, int trips, hipStream_t st);

#if defined(__HIPCC__)
// ------------------------------------------------------------------------------------------
// wave64 reductions.  DPP row shifts reduce inside each row of 16 lanes, the two row
// broadcasts carry the partial results to lane 63 (GFX9 DPP controls), readlane makes the
// result uniform.  Lanes whose DPP source is outside the row keep `identity`.
// ------------------------------------------------------------------------------------------
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t identity, uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp((int)identity, (int)v, CTRL, ROW_MASK, 0xf, false);
}

__device__ __forceinline__ uint32_t wave_min_u32(uint32_t x)
{
    const uint32_t id = 0xFFFFFFFFu;
    uint32_t v = x;
    v = min(v, dpp_u32<0x111, 0xf>(id, v));   // row_shr:1
    v = min(v, dpp_u32<0x112, 0xf>(id, v));   // row_shr:2
    v = min(v, dpp_u32<0x114, 0xf>(id, v));   // row_shr:4
    v = min(v, dpp_u32<0x118, 0xf>(id, v));   // row_shr:8
    v = min(v, dpp_u32<0x142, 0xa>(id, v));   // row_bcast:15 into rows 1 and 3
    v = min(v, dpp_u32<0x143, 0xc>(id, v));   // row_bcast:31 into rows 2 and 3
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t x)
{
    const uint32_t id = 0u;
    uint32_t v = x;
    v = max(v, dpp_u32<0x111, 0xf>(id, v));
    v = max(v, dpp_u32<0x112, 0xf>(id, v));
    v = max(v, dpp_u32<0x114, 0xf>(id, v));
    v = max(v, dpp_u32<0x118, 0xf>(id, v));
    v = max(v, dpp_u32<0x142, 0xa>(id, v));
    v = max(v, dpp_u32<0x143, 0xc>(id, v));
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t x)
{
    const uint32_t id = 0u;
    uint32_t v = x;
    v += dpp_u32<0x111, 0xf>(id, v);
    v += dpp_u32<0x112, 0xf>(id, v);
    v += dpp_u32<0x114, 0xf>(id, v);
    v += dpp_u32<0x118, 0xf>(id, v);
    v += dpp_u32<0x142, 0xa>(id, v);
    v += dpp_u32<0x143, 0xc>(id, v);
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// lexicographic minimum of (hi, lo) pairs over the wave: ties on hi resolved by the lowest lo
__device__ __forceinline__ void wave_min_pair_u32(uint32_t &hi, uint32_t &lo)
{
    uint32_t mh = wave_min_u32(hi);
    uint32_t ml = wave_min_u32(hi == mh ? lo : 0xFFFFFFFFu);
    hi = mh;
    lo = ml;
}

__device__ __forceinline__ uint64_t wave_min_u64(uint64_t x)
{
    uint32_t hi = (uint32_t)(x >> 32), lo = (uint32_t)x;
    wave_min_pair_u32(hi, lo);
    return ((uint64_t)hi << 32) | lo;
}

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & 63); }
#endif

}  // namespace mmbp
