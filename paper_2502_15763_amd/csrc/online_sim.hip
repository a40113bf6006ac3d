// Iteration-level online simulator: one wavefront per scenario, lane = client slot (up to four slots
// per lane when the batch size exceeds the wave).
// Decision rule of the paper's section "Online requests and iteration scheduling": with
// C_p = a_prefill * P + c_prefill the cost of the prefill that could be dispatched now and C_d the
// decode time accumulated since the last prefill, C_p >= C_d continues decoding, otherwise the
// prefill runs.  Iteration times follow the affine model of section "Experiment settings and
// baseline".  Every scalar of the state (time, C_d, counters, queue head) is wave-uniform; the
// per-request remaining tokens live in the lanes' registers.
#include "mmbp_dev.hpp"

#include "sim_trace.hpp"

namespace mmbp {
namespace {

constexpr int kBlock = 256;

// Q = client slots per lane: the batch size |J| may exceed one wave (the paper's node runs about 200
// clients), so slot c lives in lane c % 64, register c / 64.
// FAST = the host saw that no trace records are wanted and that a_prefill and b_decode fit 31 bits: the
// trace-store code is absent and the products of the time model take 32 x 64-bit multiplies.  The kernel
// is bound by instruction issue, the scalar and the vector unit about equally loaded, so both count.
template <int Q, bool FAST>
__global__ __launch_bounds__(kBlock) void online_sim_kernel(
    const int64_t *__restrict__ arrival_all, const int32_t *__restrict__ in_all, const int32_t *__restrict__ out_all,
    int S, int N, mmbp_sim_params p, int64_t *finish_all, int64_t *total_us, int64_t *busy_slot_us,
    int32_t *n_prefill_iter, int32_t *n_decode_iter, uint64_t *trace_hash, mmbp_trace_rec *trace_buf,
    int32_t *trace_len, int trace_scenarios, int trace_capacity, int32_t *status_out)
{
    constexpr int kWin = kWave * Q;            // requests per window chunk: one admission takes at most this many
    constexpr int kWinShift = Q == 1 ? 6 : Q == 2 ? 7 : 8;
    static_assert(Q == 1 || Q == 2 || Q == 4, "the window index is a mask");
    const int lane = threadIdx.x & 63;
    const int s = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * (kBlock / kWave) + (threadIdx.x >> 6)));
    if (s >= S) return;
    const int64_t *arrival = arrival_all + (size_t)s * N;
    const int32_t *in_len = in_all + (size_t)s * N;
    const int32_t *out_len = out_all + (size_t)s * N;
    int64_t *finish = finish_all + (size_t)s * N;

    // Inputs are validated as they enter the window (one read of every array): nothing of a chunk is
    // used before the chunk has been checked, and a scenario found invalid, however late, ends with
    // all its outputs zero.
    const int cap = p.cap;
    const int64_t maxtok = p.max_prefill_tokens;
    Trace<!FAST> tr;
    tr.h = kFnvBasis;
    tr.hc = hash_lane_init(lane);
    const bool traced = !FAST && trace_buf && s < trace_scenarios;
    tr.buf = traced ? trace_buf + (size_t)s * trace_capacity : nullptr;
    tr.cap = traced ? trace_capacity : 0;
    tr.len = 0; tr.run_open = 0; tr.run_count = 0; tr.run_t = 0; tr.run_D = 0;

    // The queue is consumed in order: a window of two chunks per wave is kept in LDS (the chunk that
    // holds the queue head and the one after it), so the dependent reads of every admission are LDS
    // reads; a chunk is fetched from memory once, when the head enters the chunk before it.
    __shared__ int64_t win_arr[kBlock / kWave][2 * kWin];
    __shared__ int32_t win_in[kBlock / kWave][2 * kWin], win_out[kBlock / kWave][2 * kWin];
    const int w = threadIdx.x >> 6;
    bool invalid = false;
    auto load_chunk = [&](int chunk) {
        int bad = 0;
#pragma unroll
        for (int q = 0; q < Q; q++) {
            const int i = chunk * kWin + q * kWave + lane, slot = i & (2 * kWin - 1);
            const bool in = i < N;
            const int64_t a = in ? arrival[i] : INT64_MAX;
            const int32_t li = in ? in_len[i] : 1, lo = in ? out_len[i] : 1;
            // arrival times must not decrease: the previous request's comes from the neighbouring lane, for
            // lane 0 from memory (the same cache line, or the previous one)
            int64_t prev = __shfl_up((long long)a, 1);
            if (lane == 0) prev = (in && i > 0) ? arrival[i - 1] : 0;
            if (in && (a < 0 || li < 1 || lo < 1 || a < prev)) bad = 1;
            win_arr[w][slot] = a;
            win_in[w][slot] = in ? li : 0;
            win_out[w][slot] = in ? lo : 0;
        }
        if (__any(bad)) invalid = true;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    };
    load_chunk(0);
    load_chunk(1);
    int loaded = 1;                            // highest chunk in the window

    int32_t rem[Q], rid[Q];                    // this lane's slots: remaining output tokens, request id
#pragma unroll
    for (int q = 0; q < Q; q++) { rem[q] = 0; rid[q] = 0; }
    int64_t t = 0, Cd = 0, busy = 0;
    int next = 0, done = 0, nR = 0, npre = 0, ndec = 0;
    int64_t head_arr = uniform_i64(win_arr[w][0]);

    while (done < N && !invalid) {
        const int free_slots = cap - nR;
        int nA = 0, nArr = 0;                  // admissible requests; arrived requests among the free_slots next ones
        int64_t P = 0;
        if (free_slots == 1 && head_arr <= t) {
            // one free slot (the usual case under load): the head request, which has arrived, is the admissible set
            nA = 1;
            nArr = 1;
            P = uniform_i64((int64_t)win_in[w][next & (2 * kWin - 1)]);
        } else if (free_slots > 0 && head_arr <= t) {
            // admissible set A: FCFS prefix of the arrived requests that fits the free slots and the
            // token capacity (an oversized head request is still admitted alone)
            int64_t tok[Q];
            bool arrived[Q];
#pragma unroll
            for (int q = 0; q < Q; q++) {
                const int c = q * kWave + lane, idx = next + c;
                const bool cand = c < free_slots && idx < N;
                const int slot = idx & (2 * kWin - 1);
                const int64_t arr = cand ? win_arr[w][slot] : INT64_MAX;
                arrived[q] = cand && arr <= t;
                tok[q] = arrived[q] ? (int64_t)win_in[w][slot] : 0;
                nA += __popcll(__ballot(arrived[q]));
            }
            nArr = nA;
            if (maxtok > 0 && nArr > 1) {        // (one arrived request is admitted whatever its length)
                int n2 = 0;
                int64_t carry = 0;
#pragma unroll
                for (int q = 0; q < Q; q++) {
                    const int64_t pre = carry + wave_incl_scan_tokens(tok[q]);
                    n2 += __popcll(__ballot(arrived[q] && pre <= maxtok));
                    if (Q > 1) carry = uniform_i64(__shfl((long long)pre, kWave - 1));
                }
                nA = n2 == 0 ? 1 : n2;
            }
            if (nA == 1) P = uniform_i64(tok[0]);
            else {
                int64_t mine = 0;                  // this lane's share: at most Q input lengths
#pragma unroll
                for (int q = 0; q < Q; q++) mine += q * kWave + lane < nA ? tok[q] : 0;
                P = wave_sum_tokens(mine);
            }
        }
        if (p.policy == MMBP_POLICY_PREFILL_FIRST_SINGLE && nA > 1) {      // baseline without batched prefill
            nA = 1;
            P = uniform_i64((int64_t)win_in[w][next & (2 * kWin - 1)]);
        }
        if (nA == 0 && nR == 0) {              // nothing running, nothing arrived: jump to the next arrival
            tr.other(2u, 1u, t, 0, lane);
            t = head_arr;
            continue;
        }
        bool do_prefill = false;
        int64_t Cp = 0;                        // cost of the prefill that could run now = its duration
        if (nA > 0) {
            Cp = (FAST ? mul_u32_i64((uint32_t)p.a_prefill, P) : p.a_prefill * P) + p.c_prefill;
            do_prefill = (nR == 0) || (Cp < Cd) || p.policy != MMBP_POLICY_RULE;   // baseline: prefill at once
        }
        // A prefill that fills the last free slot is followed by decode iterations whatever arrives (nothing
        // is admissible without a slot): they are applied in the same trip.
        bool decode_now = !do_prefill;
        int dA = nA, dArr = nArr, dfree = free_slots;
        if (do_prefill) {
            const int64_t dt = Cp;
            tr.other(1u, (uint32_t)nA, t, P, lane);
            t += dt;
            int base = 0;                      // free slots before this register's block
#pragma unroll
            for (int q = 0; q < Q; q++) {
                const bool is_free = q * kWave + lane < cap && rem[q] == 0;
                const uint64_t fm = __ballot(is_free);
                const int rank = base + __popcll(fm & ((1ull << lane) - 1ull));
                if (is_free && rank < nA) {
                    rid[q] = next + rank;
                    rem[q] = win_out[w][rid[q] & (2 * kWin - 1)];
                }
                base += __popcll(fm);
            }
            next += nA;
            while ((next >> kWinShift) + 1 > loaded) {     // (at most two rounds: nA <= kWin)
                loaded += 1;
                load_chunk(loaded);
            }
            nR += nA;
            // (the busy time is only read at the end: it is accumulated on the vector unit, which evens out
            //  the load of the scalar and the vector unit; the asm keeps the factor in a vector register)
            { int64_t vdt = dt; asm("" : "+v"(vdt)); busy += (int64_t)nA * vdt; }
            Cd = 0;
            { int one = 1; asm("" : "+v"(one)); npre += one; }
            head_arr = next < N ? uniform_i64(win_arr[w][next & (2 * kWin - 1)]) : INT64_MAX;
            if (nR == cap && !invalid) { decode_now = true; dA = 0; dArr = 0; dfree = 0; }
        }
        if (decode_now) {
            const int64_t D = nR;
            // decode time of the D tokens of one iteration
            const int64_t bD = FAST ? mul_u32_u32((uint32_t)p.b_decode, (uint32_t)nR) : p.b_decode * D;
            const int64_t dt = bD + p.c_decode;
            // Until a request finishes or one more request arrives that could be admitted, every boundary
            // sees the same admissible set and the same D, so the same decision: those k iterations are
            // applied at once.  With nothing admissible they run to the next finish or the next arrival
            // that finds a free slot; with a prefill waiting, also no further than the first j with
            // C_d + j * bD > C_p.
            int64_t k;
            {
                uint32_t m = 0xFFFFFFFFu;
#pragma unroll
                for (int q = 0; q < Q; q++) m = min(m, rem[q] > 0 ? (uint32_t)rem[q] : 0xFFFFFFFFu);
                k = (int64_t)wave_min_u32(m);
            }
            if (dA > 0 && bD > 0) k = min(k, uniform_i64((int64_t)udiv64((uint64_t)(Cp - Cd), (uint64_t)bD)) + 1);
            // the first request that has not arrived yet, if a slot would be free for it
            const int64_t next_arr = dArr == 0 ? head_arr
                                   : (dArr < dfree && next + dArr < N)
                                         ? uniform_i64(win_arr[w][(next + dArr) & (2 * kWin - 1)]) : INT64_MAX;
            if (dfree > 0 && next_arr != INT64_MAX && dt > 0) {
                // first boundary at or after the arrival (next_arr > t here, so the dividend is positive)
                const int64_t j = uniform_i64((int64_t)udiv64((uint64_t)(next_arr - t + dt - 1), (uint64_t)dt));
                k = min(k, max(j, (int64_t)1));
            }
            tr.decode(t, D, (uint32_t)k, lane);
            const int64_t kdt = FAST ? mul_u32_i64((uint32_t)k, dt) : k * dt;
            t += kdt;
            int nf = 0;
#pragma unroll
            for (int q = 0; q < Q; q++) {
                const bool active = rem[q] > 0;
                if (active) rem[q] -= (int32_t)k;
                const bool fin = active && rem[q] == 0;
                if (fin) finish[rid[q]] = t;
                nf += __popcll(__ballot(fin));
            }
            done += nf;
            nR -= nf;
            { int64_t vk = kdt; asm("" : "+v"(vk)); busy += D * vk; }
            Cd += FAST ? mul_u32_i64((uint32_t)k, bD) : k * bD;
            { int vk2 = (int)k; asm("" : "+v"(vk2)); ndec += vk2; }
        }
    }
    if (invalid) {
        for (int i = lane; i < N; i += kWave) finish[i] = 0;
        if (lane == 0) {
            total_us[s] = 0; busy_slot_us[s] = 0; n_prefill_iter[s] = 0; n_decode_iter[s] = 0;
            trace_hash[s] = 0;
            if (trace_len && s < trace_scenarios) trace_len[s] = 0;
            status_out[s] = MMBP_ST_BAD_SIM_INPUT;
        }
        return;
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
#define MMBP_SIM_LAUNCH(QQ, FF) \
    online_sim_kernel<QQ, FF><<<g, b, 0, st>>>(arrival_us, in_len, out_len, S, N, p, finish_us, total_us, busy_slot_us, \
                                               n_prefill_iter, n_decode_iter, trace_hash, trace_buf, trace_len, \
                                               trace_scenarios, trace_capacity, status_out)
    const bool fast = (!trace_buf || trace_scenarios <= 0) && p.a_prefill >= 0 && p.a_prefill < (1ll << 31) &&
                      p.b_decode >= 0 && p.b_decode < (1ll << 31);
    if (fast) {
        if (p.cap <= kWave) MMBP_SIM_LAUNCH(1, true);
        else if (p.cap <= 2 * kWave) MMBP_SIM_LAUNCH(2, true);
        else MMBP_SIM_LAUNCH(4, true);
    } else {
        if (p.cap <= kWave) MMBP_SIM_LAUNCH(1, false);
        else if (p.cap <= 2 * kWave) MMBP_SIM_LAUNCH(2, false);
        else MMBP_SIM_LAUNCH(4, false);
    }
#undef MMBP_SIM_LAUNCH
    return hipGetLastError();
}

}  // namespace mmbp
