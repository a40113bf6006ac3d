// Generic MMBP local search: full 64-bit arithmetic, state in global memory, one workgroup per
// scenario.  It is the path for scenarios whose loads do not narrow exactly to 32 bits; the
// LDS-resident and multi-workgroup kernels leave those scenarios marked pending and this kernel
// picks them up.  Candidate value = makespan after the candidate (MMBP objective max_j t_j):
// the two changed loads and the largest untouched load.
#include "mmbp_dev.hpp"

namespace mmbp {

namespace {

constexpr int kBlock = 256;
constexpr int kWaves = kBlock / kWave;

struct Top3 {
    int64_t v[3];
    int j[3];
};

// largest load among clients other than a and b
__device__ __forceinline__ int64_t others_max(const Top3 &t, int a, int b)
{
    if (t.j[0] != a && t.j[0] != b) return t.v[0];
    if (t.j[1] != a && t.j[1] != b) return t.v[1];
    return t.v[2];
}

__device__ __forceinline__ void take(int64_t &bv, uint64_t &bid, int64_t v, uint64_t id)
{
    if (v < bv || (v == bv && id < bid)) { bv = v; bid = id; }
}

__device__ __forceinline__ uint64_t sat_add(uint64_t a, uint64_t b)
{
    uint64_t r = a + b;
    return r >= (uint64_t)kCostSumLimit ? (uint64_t)kCostSumLimit : r;
}

template <typename CostT>
__global__ __launch_bounds__(kBlock) void ls_generic_kernel(
    const CostT *__restrict__ cost_all, int N, int M, int cap, int max_passes, int32_t *assign_all,
    int64_t *load_out, int64_t *makespan_out, int32_t *passes_out, uint64_t *evals_out,
    uint64_t *applied_log, int32_t *status_out)
{
    const int s = blockIdx.x;
    if (status_out[s] != kPending) return;
    const CostT *c = cost_all + (size_t)s * N;
    int32_t *asg = assign_all + (size_t)s * N;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    __shared__ int64_t load[MMBP_MAX_M];
    __shared__ int32_t cnt[MMBP_MAX_M];
    __shared__ int bad_cost, bad_assign;
    __shared__ uint64_t wsum[kWaves];
    __shared__ int64_t red_v[kWaves];
    __shared__ uint64_t red_id[kWaves];
    __shared__ Top3 top;
    __shared__ int passes_sh, status_sh;

    for (int j = tid; j < M; j += kBlock) { load[j] = 0; cnt[j] = 0; }
    if (tid == 0) { bad_cost = 0; bad_assign = 0; passes_sh = 0; status_sh = MMBP_ST_OK; }
    __syncthreads();

    // ---- validation, counts ----
    uint64_t part = 0;
    int my_bad_cost = 0, my_bad_assign = 0;
    for (int i = tid; i < N; i += kBlock) {
        int64_t ci = (int64_t)c[i];
        if (ci < 0 || ci >= kCostSumLimit) my_bad_cost = 1;
        else part = sat_add(part, (uint64_t)ci);
        int a = asg[i];
        if (a < 0 || a >= M) my_bad_assign = 1;
        else atomicAdd(&cnt[a], 1);
    }
    for (int off = 32; off >= 1; off >>= 1) part = sat_add(part, __shfl_xor((unsigned long long)part, off));
    if (lane == 0) wsum[wave] = part;
    if (my_bad_cost) bad_cost = 1;
    if (my_bad_assign) bad_assign = 1;
    __syncthreads();
    if (tid == 0) {
        uint64_t tot = 0;
        for (int w = 0; w < kWaves; w++) tot = sat_add(tot, wsum[w]);
        if (tot >= (uint64_t)kCostSumLimit) bad_cost = 1;
        if (!bad_assign)
            for (int j = 0; j < M; j++) if (cnt[j] > cap) bad_assign = 1;
    }
    __syncthreads();
    if (bad_cost || bad_assign) {
        for (int j = tid; j < M; j += kBlock) load_out[(size_t)s * M + j] = 0;
        if (tid == 0) {
            makespan_out[s] = 0; passes_out[s] = 0;
            if (evals_out) evals_out[s] = 0;
            status_out[s] = bad_cost ? MMBP_ST_BAD_COST : MMBP_ST_BAD_ASSIGN;
        }
        return;
    }
    for (int i = tid; i < N; i += kBlock)
        atomicAdd((unsigned long long *)&load[asg[i]], (unsigned long long)(int64_t)c[i]);
    __syncthreads();

    uint64_t my_evals = 0;
    int my_pass = 0;
    const uint64_t NM = (uint64_t)N * (uint64_t)M;

    for (;;) {
        if (tid == 0) {
            if (passes_sh == max_passes) status_sh = MMBP_ST_TRUNCATED;
            Top3 t;
            for (int q = 0; q < 3; q++) { t.v[q] = 0; t.j[q] = -1; }
            for (int j = 0; j < M; j++) {
                int64_t l = load[j];
                if (t.j[0] < 0 || l > t.v[0]) { t.v[2] = t.v[1]; t.j[2] = t.j[1]; t.v[1] = t.v[0]; t.j[1] = t.j[0]; t.v[0] = l; t.j[0] = j; }
                else if (t.j[1] < 0 || l > t.v[1]) { t.v[2] = t.v[1]; t.j[2] = t.j[1]; t.v[1] = l; t.j[1] = j; }
                else if (t.j[2] < 0 || l > t.v[2]) { t.v[2] = l; t.j[2] = j; }
            }
            top = t;
        }
        __syncthreads();
        if (status_sh == MMBP_ST_TRUNCATED) break;
        const Top3 t = top;
        const int64_t T = t.v[0];

        int64_t bv = INT64_MAX;
        uint64_t bid = UINT64_MAX;
        for (int i = tid; i < N; i += kBlock) {
            const int a = asg[i];
            const int64_t ci = (int64_t)c[i];
            const int64_t la = load[a];
            for (int b = 0; b < M; b++) {
                if (b == a) continue;
                my_evals++;
                if (cnt[b] + 1 > cap) continue;
                int64_t v = max(max(la - ci, load[b] + ci), others_max(t, a, b));
                take(bv, bid, v, (uint64_t)i * (uint64_t)M + (uint64_t)b);
            }
            for (int k = i + 1; k < N; k++) {
                const int b = asg[k];
                if (b == a) continue;
                my_evals++;
                const int64_t d = ci - (int64_t)c[k];
                int64_t v = max(max(la - d, load[b] + d), others_max(t, a, b));
                take(bv, bid, v, NM + (uint64_t)i * (uint64_t)N + (uint64_t)k);
            }
        }
        for (int off = 32; off >= 1; off >>= 1) {
            int64_t ov = __shfl_xor((long long)bv, off);
            uint64_t oid = __shfl_xor((unsigned long long)bid, off);
            take(bv, bid, ov, oid);
        }
        if (lane == 0) { red_v[wave] = bv; red_id[wave] = bid; }
        __syncthreads();
        if (tid == 0) {
            int64_t v = red_v[0];
            uint64_t id = red_id[0];
            for (int w = 1; w < kWaves; w++) take(v, id, red_v[w], red_id[w]);
            if (id != UINT64_MAX && v < T) {
                if (id < NM) {
                    int i = (int)(id / (uint64_t)M), b = (int)(id % (uint64_t)M);
                    int a = asg[i];
                    int64_t ci = (int64_t)c[i];
                    load[a] -= ci; load[b] += ci;
                    cnt[a]--; cnt[b]++;
                    asg[i] = b;
                } else {
                    uint64_t r = id - NM;
                    int i = (int)(r / (uint64_t)N), k = (int)(r % (uint64_t)N);
                    int a = asg[i], b = asg[k];
                    int64_t d = (int64_t)c[i] - (int64_t)c[k];
                    load[a] -= d; load[b] += d;
                    asg[i] = b; asg[k] = a;
                }
                if (applied_log) applied_log[(size_t)s * max_passes + passes_sh] = id;
                passes_sh++;
            }
            __threadfence_block();
        }
        __syncthreads();
        if (passes_sh == my_pass) break;   // nothing applied: local optimum
        my_pass = passes_sh;
    }

    // ---- write back ----
    for (int off = 32; off >= 1; off >>= 1) my_evals += __shfl_xor((unsigned long long)my_evals, off);
    if (lane == 0) wsum[wave] = my_evals;
    __syncthreads();
    for (int j = tid; j < M; j += kBlock) load_out[(size_t)s * M + j] = load[j];
    if (tid == 0) {
        int64_t T = 0;
        for (int j = 0; j < M; j++) T = max(T, load[j]);
        makespan_out[s] = T;
        passes_out[s] = passes_sh;
        uint64_t e = 0;
        for (int w = 0; w < kWaves; w++) e += wsum[w];
        if (evals_out) evals_out[s] = e;
        status_out[s] = status_sh;
    }
}

}  // namespace

hipError_t launch_ls_generic(const void *cost, int dtype, int S, int N, int M, int cap, int max_passes,
                             int32_t *assign, int64_t *load_out, int64_t *makespan_out, int32_t *passes_out,
                             uint64_t *evals_out, uint64_t *applied_log, int32_t *status_out, hipStream_t st)
{
    if (dtype == MMBP_I32)
        ls_generic_kernel<int32_t><<<dim3(S), dim3(kBlock), 0, st>>>(
            (const int32_t *)cost, N, M, cap, max_passes, assign, load_out, makespan_out, passes_out, evals_out,
            applied_log, status_out);
    else
        ls_generic_kernel<int64_t><<<dim3(S), dim3(kBlock), 0, st>>>(
            (const int64_t *)cost, N, M, cap, max_passes, assign, load_out, makespan_out, passes_out, evals_out,
            applied_log, status_out);
    return hipGetLastError();
}

}  // namespace mmbp
