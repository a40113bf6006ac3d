// Iteration-level simulator fed by an offline assignment: one wavefront per scenario, lane = client.
//
// Request scheduling follows the sorting and online preemptive method of the paper's section
// "Online requests and iteration scheduling": I_j = the requests assigned to client j, sorted by
// N^p_i + N^d_i, longest first (equal lengths: lower index first); remain_token(j) = sum of the
// lengths left in I_j.  At an iteration boundary the clients are visited in index order; an idle
// client takes the head of its own I_j if there is one, otherwise the head of the I_v of the client
// v with the largest positive remain_token (lowest v among equals).  The requests picked this way
// form the prefill that could be dispatched (cut by the prefill token cap like the FCFS prefix);
// the iteration decision and the time model are those of the FCFS simulator, and picks are only
// taken when the prefill is dispatched.  All requests are known at t = 0.
//
// Layout: the sorted queues sit one after the other in LDS (request index u16 and length u32 per
// position); a lane keeps the head / end of its queue, its remain_token and its running request
// in registers; time, C_d and the counters are wave-uniform.
#include "mmbp_dev.hpp"

#include "sim_trace.hpp"

namespace mmbp {
namespace {

__device__ __forceinline__ int64_t readlane_i64(int64_t x, int l)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)x, l);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)((uint64_t)x >> 32), l);
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

__global__ __launch_bounds__(kWave) void online_sim_assigned_kernel(
    const int32_t *__restrict__ in_all, const int32_t *__restrict__ out_all, const int32_t *__restrict__ assign_all,
    int S, int N, mmbp_sim_params p, int64_t *finish_all, int64_t *total_us, int64_t *busy_slot_us,
    int32_t *n_prefill_iter, int32_t *n_decode_iter, uint64_t *trace_hash, int32_t *served_all, int64_t *start_all,
    mmbp_trace_rec *trace_buf, int32_t *trace_len, int trace_scenarios, int trace_capacity, int32_t *status_out)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    uint32_t *qlen = reinterpret_cast<uint32_t *>(lds_raw);                 // [N] length of the request at a queue position
    uint16_t *order = reinterpret_cast<uint16_t *>(lds_raw + 4 * (size_t)N); // [N] request index at a queue position
    __shared__ int cursor[kWave];

    const int lane = threadIdx.x;
    const int s = blockIdx.x;
    if (s >= S) return;
    const int32_t *in_len = in_all + (size_t)s * N;
    const int32_t *out_len = out_all + (size_t)s * N;
    const int32_t *assign = assign_all + (size_t)s * N;
    int64_t *finish = finish_all + (size_t)s * N;
    int32_t *served_by = served_all ? served_all + (size_t)s * N : nullptr;
    int64_t *start_us = start_all ? start_all + (size_t)s * N : nullptr;
    const int cap = p.cap;

    // ---- validation ----
    int bad = 0;
    for (int i = lane; i < N; i += kWave) {
        const int a = assign[i];
        if (in_len[i] < 1 || out_len[i] < 1 || a < 0 || a >= cap) bad = 1;
    }
    if (__any(bad)) {
        for (int i = lane; i < N; i += kWave) {
            finish[i] = 0;
            if (served_by) served_by[i] = -1;
            if (start_us) start_us[i] = 0;
        }
        if (lane == 0) {
            total_us[s] = 0; busy_slot_us[s] = 0; n_prefill_iter[s] = 0; n_decode_iter[s] = 0;
            trace_hash[s] = 0;
            if (trace_len && s < trace_scenarios) trace_len[s] = 0;
            status_out[s] = MMBP_ST_BAD_SIM_INPUT;
        }
        return;
    }

    // ---- the sorted queues ----
    cursor[lane] = 0;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    for (int i = lane; i < N; i += kWave) atomicAdd(&cursor[assign[i]], 1);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    const int cnt = cursor[lane];
    int incl = cnt;
    for (int off = 1; off < kWave; off <<= 1) {
        const int y = __shfl_up(incl, off);
        if (lane >= off) incl += y;
    }
    const int qbeg = incl - cnt, qend = incl;
    __builtin_amdgcn_wave_barrier();
    cursor[lane] = qbeg;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    for (int i = lane; i < N; i += kWave) {
        const int pos = min(atomicAdd(&cursor[assign[i]], 1), N - 1);
        order[pos] = (uint16_t)i;
        qlen[pos] = (uint32_t)in_len[i] + (uint32_t)out_len[i];
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    int64_t remain = 0;
    for (int a = qbeg; a < qend; a++) {                  // insertion sort of this lane's queue: longest first, then index
        const uint32_t kl = qlen[a];
        const uint16_t ki = order[a];
        remain += (int64_t)kl;
        int b = a;
        while (b > qbeg) {
            const uint32_t pl = qlen[b - 1];
            const uint16_t pi = order[b - 1];
            if (pl > kl || (pl == kl && pi < ki)) break;
            qlen[b] = pl; order[b] = pi;
            b--;
        }
        qlen[b] = kl; order[b] = ki;
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();

    Trace tr;
    tr.h = kFnvBasis;
    tr.hc = hash_lane_init(lane);
    const bool traced = trace_buf && s < trace_scenarios;
    tr.buf = traced ? trace_buf + (size_t)s * trace_capacity : nullptr;
    tr.cap = traced ? trace_capacity : 0;
    tr.len = 0; tr.run_open = 0; tr.run_count = 0; tr.run_t = 0; tr.run_D = 0;

    const int64_t maxtok = p.max_prefill_tokens;
    int head = qbeg;
    int32_t rem = 0, rid = 0;                  // this client's running request: remaining output tokens, index
    int64_t t = 0, Cd = 0, busy = 0;
    int done = 0, nR = 0, npre = 0, ndec = 0;
    int status = MMBP_ST_OK;

    while (done < N) {                         // every trip starts a request or retires output tokens
        // ---- what the idle clients would take now (nothing is taken yet) ----
        const bool idle = lane < cap && rem == 0;
        const unsigned long long idle_mask = __ballot(idle);
        int pick_pos = -1, pick_src = -1;
        if (idle_mask) {
            const unsigned long long steal_mask = __ballot(idle && head >= qend);
            if (steal_mask == 0) {
                if (idle) { pick_pos = head; pick_src = lane; }          // every idle client has work of its own
            } else {
                int th = head;                                           // tentative heads and remain_token
                int64_t trm = remain;
                unsigned long long m = idle_mask;
                while (m) {
                    const int j = __builtin_ctzll(m);
                    m &= m - 1;
                    int src = -1;
                    if (__builtin_amdgcn_readlane(th, j) < __builtin_amdgcn_readlane(qend, j)) src = j;
                    else {
                        const uint32_t hi = wave_max_u32((uint32_t)((uint64_t)trm >> 32));
                        const uint32_t lo = wave_max_u32((uint32_t)((uint64_t)trm >> 32) == hi ? (uint32_t)trm : 0u);
                        const int64_t mx = (int64_t)(((uint64_t)hi << 32) | lo);
                        if (mx > 0) src = __builtin_ctzll(__ballot(trm == mx));
                    }
                    if (src < 0) continue;
                    const int pos = min(max(__builtin_amdgcn_readlane(th, src), 0), N - 1);
                    const int64_t len = (int64_t)qlen[pos];
                    if (lane == j) { pick_pos = pos; pick_src = src; }
                    if (lane == src) { th += 1; trm -= len; }
                }
            }
        }
        // picks in client order, cut like the FCFS prefix by the token cap (the first always fits)
        bool pick = pick_pos >= 0;
        const int idx = pick ? (int)order[pick_pos] : 0;
        const int64_t tok = pick ? (int64_t)in_len[idx] : 0;
        const int64_t len = pick ? (int64_t)qlen[pick_pos] : 0;
        unsigned long long pick_mask = __ballot(pick);
        if (pick_mask) {
            const int first = __builtin_ctzll(pick_mask);
            if (p.policy == MMBP_POLICY_PREFILL_FIRST_SINGLE) pick = pick && lane == first;
            else if (maxtok > 0) {
                const int64_t pre = wave_incl_scan_i64(tok, lane);
                const unsigned long long fail = __ballot(pick && lane != first && pre > maxtok);
                if (fail) pick = pick && lane < __builtin_ctzll(fail);
            }
            pick_mask = __ballot(pick);
        }
        const int nA = __popcll(pick_mask);
        const int64_t P = nA == 0 ? 0 : wave_sum_i64(pick ? tok : 0);
        if (nA == 0 && nR == 0) { status = MMBP_ST_BAD_SIM_INPUT; break; }      // cannot happen while requests are left

        bool do_prefill = false;
        if (nA > 0) {
            const int64_t Cp = p.a_prefill * P + p.c_prefill;
            do_prefill = (nR == 0) || (Cp < Cd) || p.policy != MMBP_POLICY_RULE;
        }
        if (do_prefill) {
            const int64_t dt = p.a_prefill * P + p.c_prefill;
            tr.other(1u, (uint32_t)nA, t, P, lane);
            if (pick) {
                rid = idx;
                rem = (int32_t)(len - tok);
                if (served_by) served_by[idx] = lane;
                if (start_us) start_us[idx] = t;
            }
            unsigned long long m = pick_mask;                // the queues the picks came from move on
            while (m) {
                const int j = __builtin_ctzll(m);
                m &= m - 1;
                const int src = __builtin_amdgcn_readlane(pick_src, j);
                const int64_t lj = readlane_i64(len, j);
                if (lane == src) { head += 1; remain -= lj; }
            }
            t += dt;
            nR += nA;
            busy += (int64_t)nA * dt;
            Cd = 0;
            npre++;
        } else {
            const int64_t D = nR;
            const int64_t bD = p.b_decode * D;              // decode time of the D tokens of one iteration
            const int64_t dt = bD + p.c_decode;
            int64_t k = 1;                                   // nothing to pick: straight to the next finish
            if (nA == 0) k = (int64_t)wave_min_u32(rem > 0 ? (uint32_t)rem : 0xFFFFFFFFu);
            tr.decode(t, D, (uint32_t)k, lane);
            const int64_t kdt = k * dt;
            t += kdt;
            const bool active = rem > 0;
            if (active) rem -= (int32_t)k;
            const bool fin = active && rem == 0;
            if (fin) finish[rid] = t;
            const int nf = __popcll(__ballot(fin));
            done += nf;
            nR -= nf;
            busy += D * kdt;
            Cd += k * bD;
            ndec += (int)k;
        }
    }
    tr.flush(lane);
    if (lane == 0) {
        total_us[s] = t; busy_slot_us[s] = busy; n_prefill_iter[s] = npre; n_decode_iter[s] = ndec;
        trace_hash[s] = tr.h;
        if (trace_len && s < trace_scenarios) trace_len[s] = tr.len;
        status_out[s] = status;
    }
}

}  // namespace

size_t sim_assigned_lds_bytes(int N) { return 6 * (size_t)N + 16; }

hipError_t launch_online_sim_assigned(const int32_t *in_len, const int32_t *out_len, const int32_t *assign, int S, int N,
                                      const mmbp_sim_params &p, int64_t *finish_us, int64_t *total_us,
                                      int64_t *busy_slot_us, int32_t *n_prefill_iter, int32_t *n_decode_iter,
                                      uint64_t *trace_hash, int32_t *served_by, int64_t *start_us,
                                      mmbp_trace_rec *trace_buf, int32_t *trace_len, int trace_scenarios,
                                      int trace_capacity, int32_t *status_out, hipStream_t st)
{
    online_sim_assigned_kernel<<<dim3(S), dim3(kWave), sim_assigned_lds_bytes(N), st>>>(
        in_len, out_len, assign, S, N, p, finish_us, total_us, busy_slot_us, n_prefill_iter, n_decode_iter, trace_hash,
        served_by, start_us, trace_buf, trace_len, trace_scenarios, trace_capacity, status_out);
    return hipGetLastError();
}

}  // namespace mmbp
