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

template <int NBYTES>
__device__ __forceinline__ uint64_t fnv_plain(uint64_t h, uint64_t w)
{
#pragma unroll
    for (int b = 0; b < NBYTES; b++) {
        h = (h ^ (w & 0xffull)) * kFnvPrime;
        w >>= 8;
    }
    return h;
}

// FNV-1a of one 24-byte trace record (kind u32, count u32, t_start i64, x i64, little endian).
//
// A byte step is (hi:lo) <- ((hi:lo) ^ b) * prime.  The xor only touches lo, and a run of z zero
// bytes is one multiplication by prime^z, so every step has the form
//     v = lo ^ b;   lo' = v * Pl;   hi' = hi * Pl + v * Ph + mulhi(v, Pl)      (Ph:Pl = prime^z)
// The lo chain is the only sequential part (scalar: xor, multiply).  hi is linear in the v of the
// steps: hi_end = hi_0 * prod(Pl) + sum_s e_s * W_s,  e_s = v_s * Ph_s + mulhi(v_s, Pl_s),
// W_s = product of the Pl of the later steps, so lane s takes v_s and one 16-lane sum finishes the
// record.  Trace fields are small numbers in wide words; for count < 2^16, 0 <= t_start < 2^40 and
// 0 <= x < 2^16 the record is the fixed sequence of 14 steps below (bytes known to be zero are
// folded into runs).  Anything else takes the byte-by-byte path.
constexpr uint64_t fnv_pow(int z) { uint64_t r = 1; for (int i = 0; i < z; i++) r *= kFnvPrime; return r; }
constexpr int kHashSteps = 14;
constexpr int kStepBytes[kHashSteps] = {1, 3, 1, 1, 2, 1, 1, 1, 1, 1, 3, 1, 1, 6};   // kind, 0*3, count*2, 0*2, t*5, 0*3, x*2, 0*6
constexpr int step_after(int s) { int n = 24; for (int i = 0; i <= s; i++) n -= kStepBytes[i]; return n; }

struct HashLane {          // per-lane constants of the record hash (lane s = step s; zero beyond the steps)
    uint32_t pl, ph, w;
};

__device__ __forceinline__ HashLane hash_lane_init(int lane)
{
    HashLane c;
    c.pl = 0; c.ph = 0; c.w = 0;
#pragma unroll
    for (int st = 0; st < kHashSteps; st++)
        if (lane == st) {
            c.pl = (uint32_t)fnv_pow(kStepBytes[st]);
            c.ph = (uint32_t)(fnv_pow(kStepBytes[st]) >> 32);
            c.w = (uint32_t)fnv_pow(step_after(st));
        }
    return c;
}

__device__ __forceinline__ uint64_t fnv_record(uint64_t h, uint32_t kind, uint32_t count, int64_t t_start, int64_t x,
                                               const HashLane &c, int lane)
{
    const uint64_t ut = (uint64_t)t_start, ux = (uint64_t)x;
    if (((uint64_t)(count >> 16) | (ut >> 40) | (ux >> 16) | (uint64_t)(kind >> 8)) != 0) {
        h = fnv_plain<8>(h, (uint64_t)kind | ((uint64_t)count << 32));
        h = fnv_plain<8>(h, ut);
        return fnv_plain<8>(h, ux);
    }
    uint32_t lo = (uint32_t)h, hi = (uint32_t)(h >> 32);
    uint32_t vv = 0;
    constexpr uint32_t kP1 = (uint32_t)fnv_pow(1), kP2 = (uint32_t)fnv_pow(2), kP3 = (uint32_t)fnv_pow(3),
                       kP6 = (uint32_t)fnv_pow(6), kP24 = (uint32_t)fnv_pow(24);
    int st = 0;
    auto byte_step = [&](uint32_t b) {
        const uint32_t v = lo ^ b;
        vv = lane == st ? v : vv;
        lo = v * kP1;
        st++;
    };
    auto run_step = [&](uint32_t pl) {
        vv = lane == st ? lo : vv;
        lo = lo * pl;
        st++;
    };
    const uint32_t tl = (uint32_t)ut, th = (uint32_t)(ut >> 32);
    byte_step(kind);
    run_step(kP3);
    byte_step(count & 0xffu);
    byte_step(count >> 8);
    run_step(kP2);
    byte_step(tl & 0xffu);
    byte_step((tl >> 8) & 0xffu);
    byte_step((tl >> 16) & 0xffu);
    byte_step(tl >> 24);
    byte_step(th);
    run_step(kP3);
    byte_step((uint32_t)ux & 0xffu);
    byte_step((uint32_t)ux >> 8);
    run_step(kP6);
    uint32_t e = (vv * c.ph + __umulhi(vv, c.pl)) * c.w;
    e += dpp_u32<0x111, 0xf>(0u, e);           // sum over the first row of 16 lanes
    e += dpp_u32<0x112, 0xf>(0u, e);
    e += dpp_u32<0x114, 0xf>(0u, e);
    e += dpp_u32<0x118, 0xf>(0u, e);
    hi = hi * kP24 + (uint32_t)__builtin_amdgcn_readlane((int)e, 15);
    return ((uint64_t)hi << 32) | lo;
}

struct Trace {
    uint64_t h;
    HashLane hc;
    mmbp_trace_rec *buf;
    int cap, len;
    int run_open;
    uint32_t run_count;
    int64_t run_t, run_D;

    __device__ __forceinline__ void emit(uint32_t kind, uint32_t count, int64_t t_start, int64_t x, int lane)
    {
        h = fnv_record(h, kind, count, t_start, x, hc, lane);
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
    // k consecutive decode iterations with D running requests, the first starting at t
    __device__ __forceinline__ void decode(int64_t t, int64_t D, uint32_t k, int lane)
    {
        if (run_open && run_D == D) { run_count += k; return; }
        flush(lane);
        run_open = 1; run_count = k; run_t = t; run_D = D;
    }
    __device__ __forceinline__ void other(uint32_t kind, uint32_t count, int64_t t, int64_t x, int lane)
    {
        flush(lane);
        emit(kind, count, t, x, lane);
    }
};

__global__ __launch_bounds__(kBlock, 8) void online_sim_kernel(
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
    tr.hc = hash_lane_init(lane);
    const bool traced = trace_buf && s < trace_scenarios;
    tr.buf = traced ? trace_buf + (size_t)s * trace_capacity : nullptr;
    tr.cap = traced ? trace_capacity : 0;
    tr.len = 0; tr.run_open = 0; tr.run_count = 0; tr.run_t = 0; tr.run_D = 0;

    // The queue is consumed in order: a window of two 64-request chunks per wave is kept in LDS
    // (the chunk that holds the queue head and the one after it), so the dependent reads of every
    // admission are LDS reads; a chunk is fetched from memory once, when the head enters the chunk
    // before it.
    __shared__ int64_t win_arr[kBlock / kWave][2 * kWave];
    __shared__ int32_t win_in[kBlock / kWave][2 * kWave], win_out[kBlock / kWave][2 * kWave];
    const int w = threadIdx.x >> 6;
    auto load_chunk = [&](int chunk) {
        const int i = chunk * kWave + lane, slot = i & (2 * kWave - 1);
        const bool in = i < N;
        win_arr[w][slot] = in ? arrival[i] : INT64_MAX;
        win_in[w][slot] = in ? in_len[i] : 0;
        win_out[w][slot] = in ? out_len[i] : 0;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    };
    load_chunk(0);
    load_chunk(1);
    int loaded = 1;                            // highest chunk in the window

    int32_t rem = 0, rid = 0;                  // this lane's slot: remaining output tokens, request id
    int64_t t = 0, Cd = 0, busy = 0;
    int next = 0, done = 0, nR = 0, npre = 0, ndec = 0;
    int64_t head_arr = uniform_i64(win_arr[w][0]);

    while (done < N) {
        const int free_slots = cap - nR;
        int nA = 0;
        int64_t P = 0;
        if (free_slots > 0 && head_arr <= t) {
            // admissible set A: FCFS prefix of the arrived requests that fits the free slots and the
            // token capacity (an oversized head request is still admitted alone)
            const int idx = next + lane;
            const bool cand = lane < free_slots && idx < N;
            const int slot = idx & (2 * kWave - 1);
            const int64_t arr = cand ? win_arr[w][slot] : INT64_MAX;
            const bool arrived = cand && arr <= t;
            const int64_t tok = arrived ? (int64_t)win_in[w][slot] : 0;
            nA = __popcll(__ballot(arrived));
            if (maxtok > 0) {
                const int64_t pre = wave_incl_scan_i64(tok, lane);
                int n2 = __popcll(__ballot(arrived && pre <= maxtok));
                nA = n2 == 0 ? 1 : n2;
            }
            P = nA == 1 ? uniform_i64(tok) : wave_sum_i64(lane < nA ? tok : 0);
        }
        if (p.policy == MMBP_POLICY_PREFILL_FIRST_SINGLE && nA > 1) {      // baseline without batched prefill
            nA = 1;
            P = uniform_i64((int64_t)win_in[w][next & (2 * kWave - 1)]);
        }
        if (nA == 0 && nR == 0) {              // nothing running, nothing arrived: jump to the next arrival
            tr.other(2u, 1u, t, 0, lane);
            t = head_arr;
            continue;
        }
        bool do_prefill = false;
        if (nA > 0) {
            const int64_t Cp = p.a_prefill * P + p.c_prefill;
            do_prefill = (nR == 0) || (Cp < Cd) || p.policy != MMBP_POLICY_RULE;   // baseline: prefill at once
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
                rem = win_out[w][rid & (2 * kWave - 1)];
            }
            next += nA;
            while ((next >> 6) + 1 > loaded) {     // (at most two rounds: nA <= 64)
                loaded += 1;
                load_chunk(loaded);
            }
            nR += nA;
            busy += (int64_t)nA * dt;
            Cd = 0;
            npre++;
            head_arr = next < N ? uniform_i64(win_arr[w][next & (2 * kWave - 1)]) : INT64_MAX;
        } else {
            const int64_t D = nR;
            const int64_t dt = p.b_decode * D + p.c_decode;
            // With nothing admissible, every boundary up to the next finish or the next arrival that
            // finds a free slot takes the same decision with the same D: those k iterations are
            // applied at once.  Otherwise (a prefill is waiting for C_d to pass C_p) one at a time.
            int64_t k = 1;
            if (nA == 0) {
                k = (int64_t)wave_min_u32(rem > 0 ? (uint32_t)rem : 0xFFFFFFFFu);
                if (free_slots > 0 && head_arr != INT64_MAX && dt > 0) {
                    const int64_t j = (head_arr - t + dt - 1) / dt;      // first boundary at or after the arrival
                    k = min(k, max(j, (int64_t)1));
                }
            }
            tr.decode(t, D, (uint32_t)k, lane);
            t += k * dt;
            const bool active = rem > 0;
            if (active) rem -= (int32_t)k;
            const bool fin = active && rem == 0;
            if (fin) finish[rid] = t;
            const int nf = __popcll(__ballot(fin));
            done += nf;
            nR -= nf;
            busy += k * D * dt;
            Cd += k * p.b_decode * D;
            ndec += (int)k;
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
