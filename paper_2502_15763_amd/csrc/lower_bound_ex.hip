// Extended theoretical lower bound T^LB = t^p* + t^d* (paper section "Offline requests scheduling &
// theoretical lower bound"): more relaxation bounds on t^d* and a level table for t^p*.
//   L1 = ceil(sum T_i / M), L2 = T_(1)
//   L3(k) = T_(kM+1) + ... + T_(kM+1-k): of the kM+1 largest requests some client holds k+1
//   Lcap  = sum of the n* smallest costs, n* = the largest number of requests the per-client
//           cardinality limits force onto one client (computed on the host from cap[])
//   t^p*  = the paper's floor form on the largest level, or the cover relaxation over all levels
// One workgroup per scenario.  L3(k) needs the R = K*M + 1 largest costs in order (K = number of
// terms): their threshold T_(R) comes from a bisection on the value (the count of costs >= x is
// monotone in x), the costs above it are gathered into LDS, the rest of the R slots take the
// threshold itself, a bitonic sort orders them and a prefix sum turns every L3(k) into a difference
// of two entries.  Lcap needs one more order statistic and the sum above it (same bisection).
#include "mmbp_dev.hpp"

namespace mmbp {
namespace {

constexpr int kBlock = 1024;
constexpr int kWaves = kBlock / kWave;

struct Levels {
    int n, form;
    int64_t ncap[MMBP_LB_MAX_LEVELS], tp[MMBP_LB_MAX_LEVELS];
};

struct Red {                         // LDS scratch of the workgroup reductions
    unsigned long long a[kWaves], b[kWaves];
    int c[kWaves];
};

__device__ __forceinline__ unsigned long long sat62(unsigned long long a, unsigned long long b)
{
    const unsigned long long r = a + b;
    return r >= (unsigned long long)kCostSumLimit ? (unsigned long long)kCostSumLimit : r;
}

__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long v)
{
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

// sum over the workgroup of (cnt, sum) pairs; every thread gets the totals
__device__ void block_count_sum(Red &red, int &cnt, unsigned long long &sum)
{
    const int tid = threadIdx.x;
    const int wc = (int)wave_sum_u32((uint32_t)cnt);
    const unsigned long long ws = wave_sum_u64(sum);
    __syncthreads();                                     // earlier readers of red are done
    if ((tid & 63) == 0) { red.c[tid >> 6] = wc; red.a[tid >> 6] = ws; }
    __syncthreads();
    int tc = 0;
    unsigned long long ts = 0;
#pragma unroll
    for (int w = 0; w < kWaves; w++) { tc += red.c[w]; ts += red.a[w]; }
    cnt = tc; sum = ts;
}

// number of costs >= x (cnt) over the scenario
template <typename CostT>
__device__ int count_ge(Red &red, const CostT *__restrict__ c, int N, int64_t x)
{
    int n = 0;
    for (int i = threadIdx.x; i < N; i += kBlock) n += ((int64_t)c[i] >= x) ? 1 : 0;
    unsigned long long dummy = 0;
    block_count_sum(red, n, dummy);
    return n;
}

// r-th largest cost (1 <= r <= N), given the largest cost
template <typename CostT>
__device__ int64_t rth_largest(Red &red, const CostT *__restrict__ c, int N, int r, int64_t cmax)
{
    int64_t lo = 0, hi = cmax;                           // count_ge(lo) >= r; the answer is in [lo, hi]
    while (lo < hi) {
        const int64_t mid = lo + ((hi - lo + 1) >> 1);
        if (count_ge<CostT>(red, c, N, mid) >= r) lo = mid;
        else hi = mid - 1;
    }
    return lo;
}

template <typename CostT>
__global__ __launch_bounds__(kBlock) void lower_bound_ex_kernel(const CostT *__restrict__ cost_all, int N, int M, int K,
                                                                int nstar, const int32_t *__restrict__ prefill_tokens,
                                                                Levels lv, int64_t *lb_out, int64_t *parts_out,
                                                                int32_t *status_out)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    int64_t *top = reinterpret_cast<int64_t *>(lds_raw);  // P2 entries, P2 = the power of two at or above K*M + 1
    __shared__ Red red;
    __shared__ int s_fill;
    __shared__ unsigned long long s_carry[kWaves];
    const int s = blockIdx.x;
    const CostT *c = cost_all + (size_t)s * N;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // ---- sum, largest cost, validity, tokens ----
    unsigned long long part = 0, mx = 0, tok = 0;
    int bad = 0;
    for (int i = tid; i < N; i += kBlock) {
        int64_t ci = (int64_t)c[i];
        if (ci < 0 || ci >= kCostSumLimit) { bad = 1; ci = 0; }
        part = sat62(part, (unsigned long long)ci);
        mx = max(mx, (unsigned long long)ci);
    }
    const bool with_tp = prefill_tokens != nullptr && lv.n > 0;
    if (with_tp)
        for (int i = tid; i < N; i += kBlock) {
            const int32_t np = prefill_tokens[(size_t)s * N + i];
            if (np < 0) bad = 1;
            tok += (unsigned long long)(np < 0 ? 0 : np);
        }
    for (int off = 32; off >= 1; off >>= 1) {
        part = sat62(part, __shfl_xor(part, off));
        mx = max(mx, (unsigned long long)__shfl_xor(mx, off));
    }
    tok = wave_sum_u64(tok);
    bad = __any(bad);
    if (lane == 0) { red.a[wave] = part; red.b[wave] = mx; red.c[wave] = bad; s_carry[wave] = tok; }
    if (tid == 0) s_fill = 0;
    __syncthreads();
    unsigned long long sum = 0, cmax = 0, toks = 0;
    int anybad = 0;
#pragma unroll
    for (int w = 0; w < kWaves; w++) {
        sum = sat62(sum, red.a[w]);
        cmax = max(cmax, red.b[w]);
        toks += s_carry[w];
        anybad |= red.c[w];
    }
    // ---- t^p* (uniform) ----
    int64_t tps = 0;
    if (with_tp) {
        if (lv.form == 0) {
            int L = 0;
            for (int l = 1; l < lv.n; l++)
                if (lv.ncap[l] > lv.ncap[L] || (lv.ncap[l] == lv.ncap[L] && lv.tp[l] < lv.tp[L])) L = l;
            const int64_t q = (int64_t)(toks / (unsigned long long)lv.ncap[L]);
            if (lv.tp[L] > 0 && q > (kCostSumLimit - 1) / lv.tp[L]) anybad = 1;
            else tps = lv.tp[L] * q;
        } else {
            for (int l = 0; l < lv.n; l++) {
                const int64_t q = (int64_t)(toks / (unsigned long long)lv.ncap[l]);
                const int64_t r = (int64_t)(toks % (unsigned long long)lv.ncap[l]);
                if (lv.tp[l] > 0 && q > (kCostSumLimit - 1) / lv.tp[l] - 1) { anybad = 1; break; }
                const int64_t v = q * lv.tp[l] + (r * lv.tp[l] + lv.ncap[l] - 1) / lv.ncap[l];
                if (l == 0 || v < tps) tps = v;
            }
        }
    }
    if (anybad || sum >= (unsigned long long)kCostSumLimit) {
        if (tid == 0) { lb_out[s] = 0; status_out[s] = MMBP_ST_BAD_COST; }
        if (parts_out && tid < 6) parts_out[(size_t)s * 6 + tid] = 0;
        return;
    }
    const int64_t L1 = (int64_t)((sum + (unsigned long long)M - 1) / (unsigned long long)M);
    const int64_t L2 = (int64_t)cmax;

    // ---- L3(k), k = 1..K: the R = K*M + 1 largest costs, sorted, as prefix sums ----
    int64_t L3 = 0;
    int k3 = 0;
    if (K > 0) {
        const int R = K * M + 1;                          // the host guarantees R <= N and R <= MMBP_LB_RANK_LIMIT
        int P2 = 1;
        while (P2 < R) P2 <<= 1;
        const int64_t vR = rth_largest<CostT>(red, c, N, R, (int64_t)cmax);
        for (int i = tid; i < P2; i += kBlock) top[i] = i < R ? vR : -1;     // slots not taken by a larger cost hold T_(R)
        __syncthreads();
        for (int i = tid; i < N; i += kBlock) {
            const int64_t ci = (int64_t)c[i];
            if (ci > vR) {
                const int p = atomicAdd(&s_fill, 1);
                if (p < R) top[p] = ci;                   // (fewer than R costs exceed T_(R))
            }
        }
        __syncthreads();
        // bitonic sort, descending
        for (int k = 2; k <= P2; k <<= 1)
            for (int j = k >> 1; j > 0; j >>= 1) {
                for (int i = tid; i < P2; i += kBlock) {
                    const int ixj = i ^ j;
                    if (ixj > i) {
                        const int64_t a = top[i], b = top[ixj];
                        const bool desc = (i & k) == 0;
                        if (desc ? a < b : a > b) { top[i] = b; top[ixj] = a; }
                    }
                }
                __syncthreads();
            }
        // inclusive prefix sums in place: each thread a contiguous run, then the runs' totals
        const int per = (R + kBlock - 1) / kBlock;
        const int b0 = min(tid * per, R), b1 = min(b0 + per, R);
        unsigned long long run = 0;
        for (int i = b0; i < b1; i++) run += (unsigned long long)top[i];
        unsigned long long incl = run;
        for (int off = 1; off < kWave; off <<= 1) {
            const unsigned long long up = __shfl_up(incl, off);
            if (lane >= off) incl += up;
        }
        if (lane == kWave - 1) s_carry[wave] = incl;
        __syncthreads();
        unsigned long long base = incl - run;
        for (int w = 0; w < wave; w++) base += s_carry[w];
        for (int i = b0; i < b1; i++) { base += (unsigned long long)top[i]; top[i] = (int64_t)base; }
        __syncthreads();
        // L3(k) = P[kM+1] - P[kM-k], P[r] = sum of the r largest = top[r-1], P[0] = 0
        unsigned long long best = 0;
        for (int k = 1 + tid; k <= K; k += kBlock) {
            const int hi = k * M + 1, lo = k * M - k;
            const unsigned long long v = (unsigned long long)top[hi - 1] - (lo > 0 ? (unsigned long long)top[lo - 1] : 0ull);
            best = max(best, v);
        }
        for (int off = 32; off >= 1; off >>= 1) best = max(best, (unsigned long long)__shfl_xor(best, off));
        __syncthreads();
        if (lane == 0) red.a[wave] = best;
        __syncthreads();
        best = 0;
#pragma unroll
        for (int w = 0; w < kWaves; w++) best = max(best, red.a[w]);
        uint32_t kmin = 0xFFFFFFFFu;                       // the smallest k that attains it
        for (int k = 1 + tid; k <= K; k += kBlock) {
            const int hi = k * M + 1, lo = k * M - k;
            const unsigned long long v = (unsigned long long)top[hi - 1] - (lo > 0 ? (unsigned long long)top[lo - 1] : 0ull);
            if (v == best) { kmin = (uint32_t)k; break; }
        }
        kmin = wave_min_u32(kmin);
        __syncthreads();
        if (lane == 0) red.c[wave] = (int)kmin;
        __syncthreads();
        kmin = 0xFFFFFFFFu;
#pragma unroll
        for (int w = 0; w < kWaves; w++) kmin = min(kmin, (uint32_t)red.c[w]);
        L3 = (int64_t)best;
        k3 = best > 0 ? (int)kmin : 0;                     // (all-zero costs: no term exceeds the initial 0)
    }

    // ---- Lcap: the nstar smallest costs = everything but the N - nstar largest ----
    int64_t Lcap = 0;
    if (nstar > 0) {
        const int r = N - nstar;
        if (r <= 0) Lcap = (int64_t)sum;
        else {
            const int64_t v = rth_largest<CostT>(red, c, N, r, (int64_t)cmax);
            int cnt = 0;
            unsigned long long sgt = 0;
            for (int i = tid; i < N; i += kBlock) {
                const int64_t ci = (int64_t)c[i];
                if (ci > v) { cnt += 1; sgt += (unsigned long long)ci; }
            }
            block_count_sum(red, cnt, sgt);
            const unsigned long long toptotal = sgt + (unsigned long long)(r - cnt) * (unsigned long long)v;
            Lcap = (int64_t)(sum - toptotal);
        }
    }
    if (tid == 0) {
        lb_out[s] = max(max(L1, L2), max(L3, Lcap)) + tps;
        status_out[s] = MMBP_ST_OK;
        if (parts_out) {
            int64_t *p = parts_out + (size_t)s * 6;
            p[0] = L1; p[1] = L2; p[2] = L3; p[3] = k3; p[4] = Lcap; p[5] = tps;
        }
    }
}

}  // namespace

hipError_t launch_lower_bound_ex(const void *cost, int dtype, int S, int N, int M, int K, int nstar,
                                 const int32_t *prefill_tokens, int n_levels, const int64_t *ncap, const int64_t *tp,
                                 int tp_form, int64_t *lb_out, int64_t *parts_out, int32_t *status_out, hipStream_t st)
{
    Levels lv;
    lv.n = n_levels; lv.form = tp_form;
    for (int l = 0; l < MMBP_LB_MAX_LEVELS; l++) { lv.ncap[l] = l < n_levels ? ncap[l] : 1; lv.tp[l] = l < n_levels ? tp[l] : 0; }
    size_t P2 = 1;
    while ((long long)P2 < (long long)K * M + 1) P2 <<= 1;
    const size_t bytes = K > 0 ? P2 * sizeof(int64_t) : 16;
    hipError_t e;
#define MMBP_LBX_LAUNCH(T) \
    do { \
        if (bytes > 48 * 1024) { \
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(&lower_bound_ex_kernel<T>), \
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)(MMBP_LB_RANK_LIMIT * sizeof(int64_t))); \
            if (e != hipSuccess) return e; \
        } \
        lower_bound_ex_kernel<T><<<dim3(S), dim3(kBlock), bytes, st>>>((const T *)cost, N, M, K, nstar, prefill_tokens, lv, \
                                                                      lb_out, parts_out, status_out); \
    } while (0)
    if (dtype == MMBP_I32) MMBP_LBX_LAUNCH(int32_t);
    else MMBP_LBX_LAUNCH(int64_t);
#undef MMBP_LBX_LAUNCH
    return hipGetLastError();
}

}  // namespace mmbp
