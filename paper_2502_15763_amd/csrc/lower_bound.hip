// Theoretical lower bound T^LB = t^p* + t^d* (paper section "Offline requests scheduling &
// theoretical lower bound").  t^d* is bounded below by max(ceil(sum T_i / M), T_(1),
// T_(M) + T_(M+1)); t^p* = T^p_L * floor(sum N^p_i / N^cap_L).  One workgroup per scenario:
// one streaming pass for sum / max / validity, then the two order statistics by bisection on
// the value (count of costs >= x is monotone in x), costs held in registers when they fit.
#include "mmbp_dev.hpp"

namespace mmbp {
namespace {

constexpr int kBlock = 256;
constexpr int kWaves = kBlock / kWave;
constexpr int kRegs = 16;   // costs cached per thread (N <= kBlock * kRegs)

__device__ __forceinline__ uint64_t sat_add62(uint64_t a, uint64_t b)
{
    uint64_t r = a + b;
    return r >= (uint64_t)kCostSumLimit ? (uint64_t)kCostSumLimit : r;
}

// number of costs >= x over the whole scenario (uniform result)
template <typename CostT, bool CACHED>
__device__ __forceinline__ int count_ge(const CostT *__restrict__ c, int N, const int64_t (&reg)[kRegs], int64_t x,
                                        int *wcnt /* LDS [kWaves] */)
{
    const int tid = threadIdx.x;
    int n = 0;
    if (CACHED) {
#pragma unroll
        for (int q = 0; q < kRegs; q++) n += (reg[q] >= x) ? 1 : 0;   // absent slots hold -1
    } else {
        for (int i = tid; i < N; i += kBlock) n += ((int64_t)c[i] >= x) ? 1 : 0;
    }
    n = (int)wave_sum_u32((uint32_t)n);
    __syncthreads();                       // previous readers of wcnt are done
    if ((tid & 63) == 0) wcnt[tid >> 6] = n;
    __syncthreads();
    int tot = 0;
#pragma unroll
    for (int w = 0; w < kWaves; w++) tot += wcnt[w];
    return tot;
}

// k-th largest cost (k >= 1, k <= N), given the maximum cost
template <typename CostT, bool CACHED>
__device__ int64_t kth_largest(const CostT *__restrict__ c, int N, const int64_t (&reg)[kRegs], int k, int64_t cmax,
                               int *wcnt)
{
    int64_t lo = 0, hi = cmax;             // invariant: count_ge(lo) >= k, answer in [lo, hi]
    while (lo < hi) {
        int64_t mid = lo + ((hi - lo + 1) >> 1);
        if (count_ge<CostT, CACHED>(c, N, reg, mid, wcnt) >= k) lo = mid;
        else hi = mid - 1;
    }
    return lo;
}

template <typename CostT, bool CACHED>
__global__ __launch_bounds__(kBlock) void lower_bound_kernel(const CostT *__restrict__ cost_all, int N, int M,
                                                             const int32_t *__restrict__ prefill_tokens,
                                                             int64_t ncap_L, int64_t tp_L, int64_t *lb_out,
                                                             int32_t *status_out)
{
    const int s = blockIdx.x;
    const CostT *c = cost_all + (size_t)s * N;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    __shared__ uint64_t wsum[kWaves];
    __shared__ uint64_t wtok[kWaves];
    __shared__ uint64_t wmax[kWaves];
    __shared__ int wbad[kWaves];
    __shared__ int wcnt[kWaves];

    int64_t reg[kRegs];
#pragma unroll
    for (int q = 0; q < kRegs; q++) reg[q] = -1;

    uint64_t part = 0, mx = 0, tok = 0;
    int bad = 0;
    if (CACHED) {
#pragma unroll
        for (int q = 0; q < kRegs; q++) {
            int i = tid + q * kBlock;
            if (i < N) {
                int64_t ci = (int64_t)c[i];
                if (ci < 0 || ci >= kCostSumLimit) { bad = 1; ci = 0; }
                reg[q] = ci;
                part = sat_add62(part, (uint64_t)ci);
                mx = max(mx, (uint64_t)ci);
            }
        }
    } else {
        for (int i = tid; i < N; i += kBlock) {
            int64_t ci = (int64_t)c[i];
            if (ci < 0 || ci >= kCostSumLimit) { bad = 1; ci = 0; }
            part = sat_add62(part, (uint64_t)ci);
            mx = max(mx, (uint64_t)ci);
        }
    }
    if (prefill_tokens && ncap_L > 0)
        for (int i = tid; i < N; i += kBlock) {
            const int32_t np = prefill_tokens[(size_t)s * N + i];
            if (np < 0) bad = 1;                       // a token count cannot be negative
            tok += (uint64_t)(np < 0 ? 0 : np);
        }
    for (int off = 32; off >= 1; off >>= 1) {
        part = sat_add62(part, __shfl_xor((unsigned long long)part, off));
        mx = max(mx, (uint64_t)__shfl_xor((unsigned long long)mx, off));
        tok += __shfl_xor((unsigned long long)tok, off);
    }
    bad = __any(bad);
    if (lane == 0) { wsum[wave] = part; wmax[wave] = mx; wtok[wave] = tok; wbad[wave] = bad; }
    __syncthreads();
    uint64_t sum = 0, cmax = 0, toks = 0;
    int anybad = 0;
#pragma unroll
    for (int w = 0; w < kWaves; w++) {
        sum = sat_add62(sum, wsum[w]);
        cmax = max(cmax, wmax[w]);
        toks += wtok[w];
        anybad |= wbad[w];
    }
    if (anybad || sum >= (uint64_t)kCostSumLimit) {
        if (tid == 0) { lb_out[s] = 0; status_out[s] = MMBP_ST_BAD_COST; }
        return;
    }
    int64_t L1 = (int64_t)((sum + (uint64_t)M - 1) / (uint64_t)M);
    int64_t L2 = (int64_t)cmax;
    int64_t L3 = 0;
    if (N >= M + 1) {
        // T_(M+1) first; T_(M) >= T_(M+1) so its search starts there
        int64_t c_m1 = kth_largest<CostT, CACHED>(c, N, reg, M + 1, (int64_t)cmax, wcnt);
        int64_t lo = c_m1, hi = (int64_t)cmax;
        while (lo < hi) {
            int64_t mid = lo + ((hi - lo + 1) >> 1);
            if (count_ge<CostT, CACHED>(c, N, reg, mid, wcnt) >= M) lo = mid;
            else hi = mid - 1;
        }
        L3 = lo + c_m1;
    }
    int64_t lbd = max(L1, max(L2, L3));
    int64_t lbp = 0;
    if (prefill_tokens && ncap_L > 0) lbp = tp_L * (int64_t)(toks / (uint64_t)ncap_L);
    if (tid == 0) { lb_out[s] = lbd + lbp; status_out[s] = MMBP_ST_OK; }
}

}  // namespace

hipError_t launch_lower_bound(const void *cost, int dtype, int S, int N, int M, const int32_t *prefill_tokens,
                              int64_t ncap_L, int64_t tp_L, int64_t *lb_out, int32_t *status_out, hipStream_t st)
{
    const bool cached = N <= kBlock * kRegs;
    dim3 g(S), b(kBlock);
#define MMBP_LB_LAUNCH(T, C) \
    lower_bound_kernel<T, C><<<g, b, 0, st>>>((const T *)cost, N, M, prefill_tokens, ncap_L, tp_L, lb_out, status_out)
    if (dtype == MMBP_I32) { if (cached) MMBP_LB_LAUNCH(int32_t, true); else MMBP_LB_LAUNCH(int32_t, false); }
    else                   { if (cached) MMBP_LB_LAUNCH(int64_t, true); else MMBP_LB_LAUNCH(int64_t, false); }
#undef MMBP_LB_LAUNCH
    return hipGetLastError();
}

}  // namespace mmbp
