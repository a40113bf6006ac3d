// Iteration-level online simulator: one wavefront per scenario, lane = client slot.
// Decision rule of the paper's section "Online requests and iteration scheduling": with
// C_p = a_prefill * P + c_prefill the cost of the prefill that could be dispatched now and C_d the
// decode time accumulated since the last prefill, C_p >= C_d continues decoding, otherwise the
// prefill runs.  Iteration times follow the affine model of section "Experiment settings and
// baseline".  Every scalar of the state (time, C_d, counters, queue head) is wave-uniform; the
// per-request remaining tokens live one per lane.
#include "mmbp_dev.hpp"

namespace mmbp {
namespace {

constexpr int kBlock = 256;
constexpr uint64_t kFnvBasis = 0xcbf29ce484222325ull;
constexpr uint64_t kFnvPrime = 0x100000001b3ull;

__device__ __forceinline__ int64_t uniform_i64(int64_t x)
{
    uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)x);
    uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uint64_t)x >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

__device__ __forceinline__ int64_t wave_sum_i64(int64_t x)
{
    for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor((long long)x, off);
    return uniform_i64(x);
}

__device__ __forceinline__ int64_t wave_incl_scan_i64(int64_t x, int lane)
{
    for (int off = 1; off < 64; off <<= 1) {
        int64_t y = __shfl_up((long long)x, off);
        if (lane >= off) x += y;
    }
    return x;
}

__device__ __forceinline__ uint64_t fnv_word(uint64_t h, uint64_t w)
{
#pragma unroll
    for (int b = 0; b < 8; b++) {
        h = (h ^ (w & 0xffull)) * kFnvPrime;
        w >>= 8;
    }
    return h;
}

struct Trace {
    uint64_t h;
    mmbp_trace_rec *buf;
    int cap, len;
    int run_open;
    uint32_t run_count;
    int64_t run_t, run_D;

    __device__ __forceinline__ void emit(uint32_t kind, uint32_t count, int64_t t_start, int64_t x, int lane)
    {
        h = fnv_word(h, (uint64_t)kind | ((uint64_t)count << 32));
        h = fnv_word(h, (uint64_t)t_start);
        h = fnv_word(h, (uint64_t)x);
        if (buf && len < cap && lane == 0) {
            mmbp_trace_rec r;
            r.kind = kind; r.count = count; r.t_start = t_start; r.x = x;
            buf[len] = r;
        }
        len++;
    }
    __device__ __forceinline__ void flush(int lane)
    {
        if (run_open) { emit(0u, run_count, run_t, run_D, lane); run_open = 0; }
    }
    __device__ __forceinline__ void decode(int64_t t, int64_t D, int lane)
    {
        if (run_open && run_D == D) { run_count++; return; }
        flush(lane);
        run_open = 1; run_count = 1; run_t = t; run_D = D;
    }
    __device__ __forceinline__ void other(uint32_t kind, uint32_t count, int64_t t, int64_t x, int lane)
    {
        flush(lane);
        emit(kind, count, t, x, lane);
    }
};

__global__ __launch_bounds__(kBlock) void online_sim_kernel(
    const int64_t *__restrict__ arrival_all, const int32_t *__restrict__ in_all, const int32_t *__restrict__ out_all,
    int S, int N, mmbp_sim_params p, int64_t *finish_all, int64_t *total_us, int64_t *busy_slot_us,
    int32_t *n_prefill_iter, int32_t *n_decode_iter, uint64_t *trace_hash, mmbp_trace_rec *trace_buf,
    int32_t *trace_len, int trace_scenarios, int trace_capacity, int32_t *status_out)
{
    const int lane = threadIdx.x & 63;
    const int s = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * (kBlock / kWave) + (threadIdx.x >> 6)));
    if (s >= S) return;
    const int64_t *arrival = arrival_all + (size_t)s * N;
    const int32_t *in_len = in_all + (size_t)s * N;
    const int32_t *out_len = out_all + (size_t)s * N;
    int64_t *finish = finish_all + (size_t)s * N;

    // ---- validation ----
    int bad = 0;
    for (int i = lane; i < N; i += kWave) {
        int64_t a = arrival[i];
        if (a < 0 || in_len[i] < 1 || out_len[i] < 1) bad = 1;
        if (i > 0 && a < arrival[i - 1]) bad = 1;
    }
    if (__any(bad)) {
        for (int i = lane; i < N; i += kWave) finish[i] = 0;
        if (lane == 0) {
            total_us[s] = 0; busy_slot_us[s] = 0; n_prefill_iter[s] = 0; n_decode_iter[s] = 0;
            trace_hash[s] = 0;
            if (trace_len && s < trace_scenarios) trace_len[s] = 0;
            status_out[s] = MMBP_ST_BAD_SIM_INPUT;
        }
        return;
    }

    const int cap = p.cap;
    const int64_t maxtok = p.max_prefill_tokens;
    Trace tr;
    tr.h = kFnvBasis;
    const bool traced = trace_buf && s < trace_scenarios;
    tr.buf = traced ? trace_buf + (size_t)s * trace_capacity : nullptr;
    tr.cap = traced ? trace_capacity : 0;
    tr.len = 0; tr.run_open = 0; tr.run_count = 0; tr.run_t = 0; tr.run_D = 0;

    int32_t rem = 0, rid = 0;                  // this lane's slot: remaining output tokens, request id
    int64_t t = 0, Cd = 0, busy = 0;
    int next = 0, done = 0, nR = 0, npre = 0, ndec = 0;
    int64_t head_arr = uniform_i64(arrival[0]);

    while (done < N) {
        const int free_slots = cap - nR;
        int nA = 0;
        int64_t P = 0;
        if (free_slots > 0 && head_arr <= t) {
            // admissible set A: FCFS prefix of the arrived requests that fits the free slots and the
            // token capacity (an oversized head request is still admitted alone)
            const int idx = next + lane;
            const bool cand = lane < free_slots && idx < N;
            const int64_t arr = cand ? arrival[idx] : INT64_MAX;
            const bool arrived = cand && arr <= t;
            const int64_t tok = arrived ? (int64_t)in_len[idx] : 0;
            nA = __popcll(__ballot(arrived));
            if (maxtok > 0) {
                const int64_t pre = wave_incl_scan_i64(tok, lane);
                int n2 = __popcll(__ballot(arrived && pre <= maxtok));
                nA = n2 == 0 ? 1 : n2;
            }
            P = wave_sum_i64(lane < nA ? tok : 0);
        }
        if (nA == 0 && nR == 0) {              // nothing running, nothing arrived: jump to the next arrival
            tr.other(2u, 1u, t, 0, lane);
            t = head_arr;
            continue;
        }
        bool do_prefill = false;
        if (nA > 0) {
            const int64_t Cp = p.a_prefill * P + p.c_prefill;
            do_prefill = (nR == 0) || (Cp < Cd);
        }
        if (do_prefill) {
            const int64_t dt = p.a_prefill * P + p.c_prefill;
            tr.other(1u, (uint32_t)nA, t, P, lane);
            t += dt;
            const bool is_free = lane < cap && rem == 0;
            const uint64_t fm = __ballot(is_free);
            const int rank = __popcll(fm & ((1ull << lane) - 1ull));
            if (is_free && rank < nA) {
                rid = next + rank;
                rem = out_len[rid];
            }
            next += nA;
            nR += nA;
            busy += (int64_t)nA * dt;
            Cd = 0;
            npre++;
            head_arr = next < N ? uniform_i64(arrival[next]) : INT64_MAX;
        } else {
            const int64_t D = nR;
            const int64_t dt = p.b_decode * D + p.c_decode;
            tr.decode(t, D, lane);
            t += dt;
            const bool active = rem > 0;
            if (active) rem -= 1;
            const bool fin = active && rem == 0;
            if (fin) finish[rid] = t;
            const int nf = __popcll(__ballot(fin));
            done += nf;
            nR -= nf;
            busy += D * dt;
            Cd += p.b_decode * D;
            ndec++;
        }
    }
    tr.flush(lane);
    if (lane == 0) {
        total_us[s] = t; busy_slot_us[s] = busy; n_prefill_iter[s] = npre; n_decode_iter[s] = ndec;
        trace_hash[s] = tr.h;
        if (trace_len && s < trace_scenarios) trace_len[s] = tr.len;
        status_out[s] = MMBP_ST_OK;
    }
}

}  // namespace

hipError_t launch_online_sim(const int64_t *arrival_us, const int32_t *in_len, const int32_t *out_len, int S, int N,
                             const mmbp_sim_params &p, int64_t *finish_us, int64_t *total_us, int64_t *busy_slot_us,
                             int32_t *n_prefill_iter, int32_t *n_decode_iter, uint64_t *trace_hash,
                             mmbp_trace_rec *trace_buf, int32_t *trace_len, int trace_scenarios, int trace_capacity,
                             int32_t *status_out, hipStream_t st)
{
    const int per_block = kBlock / kWave;
    dim3 g((S + per_block - 1) / per_block), b(kBlock);
    online_sim_kernel<<<g, b, 0, st>>>(arrival_us, in_len, out_len, S, N, p, finish_us, total_us, busy_slot_us,
                                       n_prefill_iter, n_decode_iter, trace_hash, trace_buf, trace_len,
                                       trace_scenarios, trace_capacity, status_out);
    return hipGetLastError();
}

}  // namespace mmbp
