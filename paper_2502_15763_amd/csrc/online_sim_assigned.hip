// Iteration-level simulator fed by an offline assignment: one wavefront per scenario, lane = client
// (up to four clients per lane when there are more clients than lanes).
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
// Layout: the sorted queues sit one after the other in LDS (request index u16, length u32 and, while
// every input length fits 16 bits, input length u16 per position, so that a pick reads nothing from
// global memory; 8 bytes per request keep eight scenarios of 2048 requests on a CU); a lane keeps the head / end of its queue, its remain_token and its running request
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

// Lane sl's value of register block sq (both uniform) of a per-lane array.  Every block is read with a
// constant index and the choice is made among the scalars: a select among the vector registers
// themselves was compiled into an indexed array in scratch memory, a trip to memory per steal.
template <int Q>
__device__ __forceinline__ int lane_value(const int (&a)[Q], int sq, int sl)
{
    int v = __builtin_amdgcn_readlane(a[0], sl);
#pragma unroll
    for (int q = 1; q < Q; q++) {
        const int vq = __builtin_amdgcn_readlane(a[q], sl);
        v = sq == q ? vq : v;
    }
    return v;
}

// Q = clients per lane: client j lives in lane j % 64, register j / 64 (the paper's node runs about
// 200 clients, more than one wave has lanes).
// FAST: no trace records wanted and time-model slopes below 2^31 (decided on the host), as in the FCFS simulator.
template <int Q, bool FAST>
__global__ __launch_bounds__(kWave) void online_sim_assigned_kernel(
    const int32_t *__restrict__ in_all, const int32_t *__restrict__ out_all, const int32_t *__restrict__ assign_all,
    int S, int N, mmbp_sim_params p, int64_t *finish_all, int64_t *total_us, int64_t *busy_slot_us,
    int32_t *n_prefill_iter, int32_t *n_decode_iter, uint64_t *trace_hash, int32_t *served_all, int64_t *start_all,
    mmbp_trace_rec *trace_buf, int32_t *trace_len, int trace_scenarios, int trace_capacity, int32_t *status_out)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    uint32_t *qlen = reinterpret_cast<uint32_t *>(lds_raw);                 // [N] length of the request at a queue position
    uint16_t *order = reinterpret_cast<uint16_t *>(lds_raw + 4 * (size_t)N); // [N] request index at a queue position
    uint16_t *qin = reinterpret_cast<uint16_t *>(lds_raw + 6 * (size_t)N);  // [N] its N^p_i (unused if one exceeds 16 bits)
    __shared__ int cursor[kWave * Q];

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

    auto reject = [&]() {
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
    };

    // ---- the sorted queues ----
#pragma unroll
    for (int q = 0; q < Q; q++) cursor[q * kWave + lane] = 0;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    // (inputs are validated where they are first read: the clients here, the lengths in the pass that
    //  fills the queues; nothing has been written when a scenario is rejected)
    int bad = 0, wide = 0;
    for (int i = lane; i < N; i += kWave) {
        const int a = assign[i];
        if (a < 0 || a >= cap) bad = 1;
        else atomicAdd(&cursor[a], 1);
    }
    if (__any(bad)) { reject(); return; }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    int qbeg[Q], qend[Q];
    {
        int carry = 0;                         // requests of the clients in earlier register blocks
#pragma unroll
        for (int q = 0; q < Q; q++) {
            const int cnt = cursor[q * kWave + lane];
            int incl = cnt;
            for (int off = 1; off < kWave; off <<= 1) {
                const int y = __shfl_up(incl, off);
                if (lane >= off) incl += y;
            }
            qbeg[q] = carry + incl - cnt;
            qend[q] = carry + incl;
            carry += __builtin_amdgcn_readlane(incl, kWave - 1);
        }
    }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int q = 0; q < Q; q++) cursor[q * kWave + lane] = qbeg[q];
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    for (int i = lane; i < N; i += kWave) {
        const int pos = min(atomicAdd(&cursor[assign[i]], 1), N - 1);
        const int32_t li = in_len[i], lo = out_len[i];
        if (li < 1 || lo < 1) bad = 1;
        if (li > 0xFFFF) wide = 1;
        order[pos] = (uint16_t)i;
        qlen[pos] = (uint32_t)li + (uint32_t)lo;
    }
    if (__any(bad)) { reject(); return; }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    int64_t remain[Q];
#pragma unroll
    for (int q = 0; q < Q; q++) {
        remain[q] = 0;
        for (int a = qbeg[q]; a < qend[q]; a++) {        // insertion sort of this client's queue: longest first, then index
            const uint32_t kl = qlen[a];
            const uint16_t ki = order[a];
            remain[q] += (int64_t)kl;
            int b = a;
            while (b > qbeg[q]) {
                const uint32_t pl = qlen[b - 1];
                const uint16_t pi = order[b - 1];
                if (pl > kl || (pl == kl && pi < ki)) break;
                qlen[b] = pl; order[b] = pi;
                b--;
            }
            qlen[b] = kl; order[b] = ki;
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    // While every client's remain_token is below 2^24, (remain_token, lowest client) is one 32-bit key and a
    // steal needs one wave reduction instead of three (remain_token only goes down).
    bool small_keys = true;
#pragma unroll
    for (int q = 0; q < Q; q++) small_keys = small_keys && !__any(remain[q] >= (1ll << 24));
    const bool wide_in = __any(wide);          // some N^p_i does not fit 16 bits: picks read in_len from memory
    if (!wide_in)
        for (int pos = lane; pos < N; pos += kWave) qin[pos] = (uint16_t)in_len[order[pos]];
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();

    Trace<!FAST> tr;
    tr.h = kFnvBasis;
    tr.hc = hash_lane_init(lane);
    const bool traced = !FAST && trace_buf && s < trace_scenarios;
    tr.buf = traced ? trace_buf + (size_t)s * trace_capacity : nullptr;
    tr.cap = traced ? trace_capacity : 0;
    tr.len = 0; tr.run_open = 0; tr.run_count = 0; tr.run_t = 0; tr.run_D = 0;

    const int64_t maxtok = p.max_prefill_tokens;
    int head[Q];
    int32_t rem[Q], rid[Q];                    // each client's running request: remaining output tokens, index
#pragma unroll
    for (int q = 0; q < Q; q++) { head[q] = qbeg[q]; rem[q] = 0; rid[q] = 0; }
    int64_t t = 0, Cd = 0, busy = 0;
    int done = 0, nR = 0, npre = 0, ndec = 0;
    int status = MMBP_ST_OK;

    while (done < N) {                         // every trip starts a request or retires output tokens
        // ---- what the idle clients would take now (nothing is taken yet) ----
        bool idle[Q];
        unsigned long long idle_mask[Q];
        bool any_idle = false, any_steal = false;
#pragma unroll
        for (int q = 0; q < Q; q++) {
            idle[q] = q * kWave + lane < cap && rem[q] == 0;
            idle_mask[q] = __ballot(idle[q]);
            any_idle = any_idle || idle_mask[q] != 0;
            any_steal = any_steal || __ballot(idle[q] && head[q] >= qend[q]) != 0;
        }
        int pick_pos[Q], pick_src[Q];
#pragma unroll
        for (int q = 0; q < Q; q++) { pick_pos[q] = -1; pick_src[q] = -1; }
        if (any_idle) {
            if (!any_steal) {
#pragma unroll
                for (int q = 0; q < Q; q++)
                    if (idle[q]) { pick_pos[q] = head[q]; pick_src[q] = q * kWave + lane; }   // every idle client has work of its own
            } else {
                int th[Q];                                               // tentative heads and remain_token
                int64_t trm[Q];
#pragma unroll
                for (int q = 0; q < Q; q++) { th[q] = head[q]; trm[q] = remain[q]; }
                // Only a prefix of the picks can join the prefill (one pick under the single-request baseline,
                // the picks up to the first that exceeds the token cap otherwise), and nothing is taken
                // here, so the visit ends with the pick that closes that prefix.
                int64_t acc_tok = 0;
                int npk = 0;
                bool closed = false;
#pragma unroll
                for (int jq = 0; jq < Q; jq++) {                         // the idle clients in index order
                    unsigned long long m = closed ? 0ull : idle_mask[jq];
                    while (m) {
                        const int jl = __builtin_ctzll(m);
                        m &= m - 1;
                        int src = -1;
                        if (__builtin_amdgcn_readlane(th[jq], jl) < __builtin_amdgcn_readlane(qend[jq], jl)) src = jq * kWave + jl;
                        else if (small_keys) {
                            uint32_t key = 0;                             // (remain_token, 255 - client): the maximum is the steal's source
#pragma unroll
                            for (int q = 0; q < Q; q++)
                                key = max(key, ((uint32_t)trm[q] << 8) | (uint32_t)(255 - (q * kWave + lane)));
                            const uint32_t mx = wave_max_u32(key);
                            if (mx >> 8) src = 255 - (int)(mx & 255u);
                            else {
                                closed = true;           // every queue is empty by now (lengths are positive), also for
                                m = 0;                   // the clients still to come: nobody else picks anything
                            }
                        } else {
                            int64_t bm = trm[0];                          // the largest remain_token, lowest client among equals
#pragma unroll
                            for (int q = 1; q < Q; q++) bm = max(bm, trm[q]);
                            const uint32_t hi = wave_max_u32((uint32_t)((uint64_t)bm >> 32));
                            const uint32_t lo = wave_max_u32((uint32_t)((uint64_t)bm >> 32) == hi ? (uint32_t)bm : 0u);
                            const int64_t mx = (int64_t)(((uint64_t)hi << 32) | lo);
                            if (mx > 0) {
                                uint32_t c = 0xFFFFFFFFu;
#pragma unroll
                                for (int q = Q - 1; q >= 0; q--) c = trm[q] == mx ? (uint32_t)(q * kWave + lane) : c;
                                src = (int)wave_min_u32(c);
                            } else {
                                closed = true;
                                m = 0;
                            }
                        }
                        if (src < 0) continue;
                        const int sq = src >> 6, sl = src & 63;
                        const int pos = min(max(lane_value<Q>(th, sq, sl), 0), N - 1);
                        const int64_t len = (int64_t)qlen[pos];
                        if (lane == jl) { pick_pos[jq] = pos; pick_src[jq] = src; }
                        if (lane == sl) {
#pragma unroll
                            for (int q = 0; q < Q; q++)
                                if (q == sq) { th[q] += 1; trm[q] -= len; }
                        }
                        npk++;
                        if (p.policy == MMBP_POLICY_PREFILL_FIRST_SINGLE) closed = true;
                        else if (maxtok > 0) {
                            acc_tok += wide_in ? (int64_t)in_len[order[pos]] : (int64_t)qin[pos];
                            closed = npk > 1 && acc_tok > maxtok;
                        }
                        if (closed) m = 0;
                    }
                }
            }
        }
        // picks in client order, cut like the FCFS prefix by the token cap (the first always fits)
        bool pick[Q];
        int idx[Q];
        int64_t tok[Q], len[Q];
        uint32_t first = 0xFFFFFFFFu;          // the first client that picks
        int npick = 0;
#pragma unroll
        for (int q = Q - 1; q >= 0; q--) {
            pick[q] = pick_pos[q] >= 0;
            idx[q] = pick[q] ? (int)order[pick_pos[q]] : 0;
            tok[q] = pick[q] ? (wide_in ? (int64_t)in_len[idx[q]] : (int64_t)qin[pick_pos[q]]) : 0;
            len[q] = pick[q] ? (int64_t)qlen[pick_pos[q]] : 0;
            const unsigned long long pm = __ballot(pick[q]);
            if (pm) first = (uint32_t)(q * kWave + __builtin_ctzll(pm));
            npick += __popcll(pm);
        }
        int nA = 0;
        int64_t P = 0;
        if (npick == 1) {                      // one pick (the usual case under load): it is the prefill
            int tok32[Q];
#pragma unroll
            for (int q = 0; q < Q; q++) tok32[q] = (int)tok[q];
            nA = 1;
            P = (int64_t)lane_value<Q>(tok32, (int)(first >> 6), (int)(first & 63u));
        } else if (first != 0xFFFFFFFFu) {
            if (p.policy == MMBP_POLICY_PREFILL_FIRST_SINGLE) {
#pragma unroll
                for (int q = 0; q < Q; q++) pick[q] = pick[q] && (uint32_t)(q * kWave + lane) == first;
            } else if (maxtok > 0) {
                uint32_t failpos = 0xFFFFFFFFu;  // the first pick that does not fit: it and the later ones wait
                int64_t carry = 0;
#pragma unroll
                for (int q = 0; q < Q; q++) {
                    const int64_t pre = carry + wave_incl_scan_tokens(tok[q]);
                    const unsigned long long fail = __ballot(pick[q] && (uint32_t)(q * kWave + lane) != first && pre > maxtok);
                    if (fail && failpos == 0xFFFFFFFFu) failpos = (uint32_t)(q * kWave + __builtin_ctzll(fail));
                    if (Q > 1) carry = uniform_i64(__shfl((long long)pre, kWave - 1));
                }
#pragma unroll
                for (int q = 0; q < Q; q++) pick[q] = pick[q] && (uint32_t)(q * kWave + lane) < failpos;
            }
            int64_t mine = 0;                      // this lane's share: at most Q input lengths
#pragma unroll
            for (int q = 0; q < Q; q++) {
                nA += __popcll(__ballot(pick[q]));
                mine += pick[q] ? tok[q] : 0;
            }
            P = wave_sum_tokens(mine);
        }
        if (nA == 0 && nR == 0) { status = MMBP_ST_BAD_SIM_INPUT; break; }      // cannot happen while requests are left

        bool do_prefill = false;
        int64_t Cp = 0;                        // cost of the prefill that could run now = its duration
        if (nA > 0) {
            Cp = (FAST ? mul_u32_i64((uint32_t)p.a_prefill, P) : p.a_prefill * P) + p.c_prefill;
            do_prefill = (nR == 0) || (Cp < Cd) || p.policy != MMBP_POLICY_RULE;
        }
        // A prefill after which every client is busy is followed by decode iterations (nobody can pick):
        // they are applied in the same trip.
        bool decode_now = !do_prefill;
        int dA = nA;
        if (do_prefill) {
            const int64_t dt = Cp;
            tr.other(1u, (uint32_t)nA, t, P, lane);
#pragma unroll
            for (int q = 0; q < Q; q++)
                if (pick[q]) {
                    rid[q] = idx[q];
                    rem[q] = (int32_t)(len[q] - tok[q]);
                    if (served_by) served_by[idx[q]] = q * kWave + lane;
                    if (start_us) start_us[idx[q]] = t;
                }
#pragma unroll
            for (int jq = 0; jq < Q; jq++) {                 // the queues the picks came from move on
                unsigned long long m = __ballot(pick[jq]);
                while (m) {
                    const int jl = __builtin_ctzll(m);
                    m &= m - 1;
                    const int src = __builtin_amdgcn_readlane(pick_src[jq], jl);
                    const int64_t lj = readlane_i64(len[jq], jl);
                    const int sq = src >> 6, sl = src & 63;
                    if (lane == sl) {
#pragma unroll
                        for (int q = 0; q < Q; q++)
                            if (q == sq) { head[q] += 1; remain[q] -= lj; }
                    }
                }
            }
            t += dt;
            nR += nA;
            { int64_t vdt = dt; asm("" : "+v"(vdt)); busy += (int64_t)nA * vdt; }     // (on the vector unit, as in the FCFS simulator)
            Cd = 0;
            npre++;
            if (nR == cap) { decode_now = true; dA = 0; }
        }
        if (decode_now) {
            const int64_t D = nR;
            // decode time of the D tokens of one iteration
            const int64_t bD = FAST ? mul_u32_u32((uint32_t)p.b_decode, (uint32_t)nR) : p.b_decode * D;
            const int64_t dt = bD + p.c_decode;
            // Until a request finishes, the idle clients and their picks stay what they are, so every
            // boundary sees the same C_p and the same D: with nothing to pick the decode iterations run
            // to the next finish; with a prefill waiting they run until C_d has passed C_p (the first j
            // with C_d + j * bD > C_p), or to the next finish if that comes first.
            int64_t k;
            {
                uint32_t m = 0xFFFFFFFFu;
#pragma unroll
                for (int q = 0; q < Q; q++) m = min(m, rem[q] > 0 ? (uint32_t)rem[q] : 0xFFFFFFFFu);
                k = (int64_t)wave_min_u32(m);
            }
            if (dA > 0 && bD > 0) k = min(k, uniform_i64((int64_t)udiv64((uint64_t)(Cp - Cd), (uint64_t)bD)) + 1);
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

size_t sim_assigned_lds_bytes(int N) { return 8 * (size_t)N + 16; }

hipError_t launch_online_sim_assigned(const int32_t *in_len, const int32_t *out_len, const int32_t *assign, int S, int N,
                                      const mmbp_sim_params &p, int64_t *finish_us, int64_t *total_us,
                                      int64_t *busy_slot_us, int32_t *n_prefill_iter, int32_t *n_decode_iter,
                                      uint64_t *trace_hash, int32_t *served_by, int64_t *start_us,
                                      mmbp_trace_rec *trace_buf, int32_t *trace_len, int trace_scenarios,
                                      int trace_capacity, int32_t *status_out, hipStream_t st)
{
    const size_t lds = sim_assigned_lds_bytes(N);
#define MMBP_SIMA_LAUNCH(QQ, FF) \
    do { \
        if (lds > 64 * 1024) {                           /* beyond the default limit: raise it for this kernel */ \
            const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&online_sim_assigned_kernel<QQ, FF>), \
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, \
                                                     (int)sim_assigned_lds_bytes(MMBP_SIM_ASSIGNED_MAX_N)); \
            if (e != hipSuccess) return e; \
        } \
        online_sim_assigned_kernel<QQ, FF><<<dim3(S), dim3(kWave), lds, st>>>( \
            in_len, out_len, assign, S, N, p, finish_us, total_us, busy_slot_us, n_prefill_iter, n_decode_iter, trace_hash, \
            served_by, start_us, trace_buf, trace_len, trace_scenarios, trace_capacity, status_out); \
    } while (0)
    const bool fast = (!trace_buf || trace_scenarios <= 0) && p.a_prefill >= 0 && p.a_prefill < (1ll << 31) &&
                      p.b_decode >= 0 && p.b_decode < (1ll << 31);
    if (fast) {
        if (p.cap <= kWave) MMBP_SIMA_LAUNCH(1, true);
        else if (p.cap <= 2 * kWave) MMBP_SIMA_LAUNCH(2, true);
        else MMBP_SIMA_LAUNCH(4, true);
    } else {
        if (p.cap <= kWave) MMBP_SIMA_LAUNCH(1, false);
        else if (p.cap <= 2 * kWave) MMBP_SIMA_LAUNCH(2, false);
        else MMBP_SIMA_LAUNCH(4, false);
    }
#undef MMBP_SIMA_LAUNCH
    return hipGetLastError();
}

}  // namespace mmbp
