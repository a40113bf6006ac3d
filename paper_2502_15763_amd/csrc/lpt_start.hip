// Longest-processing-time start for the MMBP model (paper section "Offline requests scheduling &
// theoretical lower bound": min max_j t_j, every request on exactly one client), with at most cap
// requests per client: the requests are taken by decreasing cost T_i (equal costs: lower index
// first) and each goes to the client with the smallest load among those with room (equal loads:
// lower client index).
//
// One workgroup per scenario.  Ordering: the keys (T_i << b) | (2^b - 1 - i), b = bits of N - 1, are
// sorted in LDS by a bitonic network (descending: larger cost first, then lower index); costs too
// large to pack (T_i >= 2^(63-b)) take a ranking by counting instead (rank_i = number of requests
// that precede i), which needs no packing.  The order leaves through order_out, which the second
// phase reads back.  Greedy phase: one wave, lane = client (up to four clients per lane), the load
// and count of a client stay in its lane's registers; per request one wave-wide lexicographic
// minimum of (load, client) over the clients with room.
#include "mmbp_dev.hpp"

namespace mmbp {
namespace {

constexpr int kBlock = 1024;
constexpr int kWaves = kBlock / kWave;
constexpr int kClientsPerLane = MMBP_MAX_M / kWave;      // 4

__device__ __forceinline__ unsigned long long sat62(unsigned long long a, unsigned long long b)
{
    const unsigned long long r = a + b;
    return r >= (unsigned long long)kCostSumLimit ? (unsigned long long)kCostSumLimit : r;
}

template <typename CostT>
__global__ __launch_bounds__(kBlock) void lpt_start_kernel(const CostT *__restrict__ cost_all, int N, int M, int cap,
                                                           int32_t *assign_all, int64_t *load_out, int32_t *order_all,
                                                           int32_t *status_out)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    unsigned long long *key = reinterpret_cast<unsigned long long *>(lds_raw);   // P2 entries
    __shared__ unsigned long long s_sum[kWaves], s_max[kWaves];
    __shared__ int s_bad[kWaves];
    const int s = blockIdx.x;
    const CostT *c = cost_all + (size_t)s * N;
    int32_t *asg = assign_all + (size_t)s * N;
    int32_t *order = order_all + (size_t)s * N;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // ---- validity, sum, largest cost ----
    unsigned long long part = 0, mx = 0;
    int bad = 0;
    for (int i = tid; i < N; i += kBlock) {
        long long ci = (long long)c[i];
        if (ci < 0 || ci >= kCostSumLimit) { bad = 1; ci = 0; }
        part = sat62(part, (unsigned long long)ci);
        mx = max(mx, (unsigned long long)ci);
    }
    for (int off = 32; off >= 1; off >>= 1) {
        part = sat62(part, __shfl_xor(part, off));
        mx = max(mx, (unsigned long long)__shfl_xor(mx, off));
    }
    bad = __any(bad);
    if (lane == 0) { s_sum[wave] = part; s_max[wave] = mx; s_bad[wave] = bad; }
    __syncthreads();
    unsigned long long sum = 0, cmax = 0;
    int anybad = 0;
#pragma unroll
    for (int w = 0; w < kWaves; w++) { sum = sat62(sum, s_sum[w]); cmax = max(cmax, s_max[w]); anybad |= s_bad[w]; }
    if (anybad || sum >= (unsigned long long)kCostSumLimit) {
        for (int i = tid; i < N; i += kBlock) { asg[i] = -1; order[i] = -1; }
        for (int j = tid; j < M; j += kBlock) load_out[(size_t)s * M + j] = 0;
        if (tid == 0) status_out[s] = MMBP_ST_BAD_COST;
        return;
    }

    // ---- the order ----
    int b = 0;
    while ((1 << b) < N) b++;                            // index bits
    const unsigned long long imask = (1ull << b) - 1ull;
    const bool packed = cmax < (1ull << (63 - b));
    int P2 = 1;
    while (P2 < N) P2 <<= 1;
    if (packed) {
        for (int i = tid; i < P2; i += kBlock)
            key[i] = i < N ? (((unsigned long long)c[i] << b) | (imask - (unsigned long long)i)) : 0ull;
        // (padding keys are 0 and sort last: a real key is 0 only for cost 0 and i = 2^b - 1, i.e. N = 2^b = P2,
        //  where there is no padding)
        __syncthreads();
        for (int k = 2; k <= P2; k <<= 1)
            for (int j = k >> 1; j > 0; j >>= 1) {
                for (int i = tid; i < P2; i += kBlock) {
                    const int ixj = i ^ j;
                    if (ixj > i) {
                        const unsigned long long x = key[i], y = key[ixj];
                        const bool desc = (i & k) == 0;
                        if (desc ? x < y : x > y) { key[i] = y; key[ixj] = x; }
                    }
                }
                __syncthreads();
            }
        for (int q = tid; q < N; q += kBlock) order[q] = (int32_t)(imask - (key[q] & imask));
    } else {
        // costs that do not pack: rank_i = #{j : T_j > T_i, or T_j == T_i and j < i}
        for (int i = tid; i < N; i += kBlock) key[i] = (unsigned long long)c[i];
        __syncthreads();
        for (int i = tid; i < N; i += kBlock) {
            const unsigned long long ci = key[i];
            int r = 0;
            for (int j = 0; j < N; j++) {
                const unsigned long long cj = key[j];
                r += (cj > ci || (cj == ci && j < i)) ? 1 : 0;
            }
            order[r] = i;
        }
    }
    __threadfence_block();
    __syncthreads();                                     // the order is complete and visible to wave 0
    if (wave != 0) return;

    // ---- greedy phase: wave 0, lane = clients lane, lane + 64, ... ----
    unsigned long long ld[kClientsPerLane];
    int cn[kClientsPerLane];
#pragma unroll
    for (int r = 0; r < kClientsPerLane; r++) { ld[r] = 0; cn[r] = 0; }
    // While no load can reach 2^24 (the largest load so far plus the largest cost stays below it), (load, client)
    // is one 32-bit key and a placement needs one wave reduction instead of three.
    unsigned long long top = 0;                          // the largest load so far
    for (int q0 = 0; q0 < N; q0 += kWave) {
        const int nb = min(kWave, N - q0);
        // this batch's requests, one per lane
        int bi = 0;
        unsigned long long bc = 0;
        if (lane < nb) {
            bi = order[q0 + lane];
            bc = packed ? (key[q0 + lane] >> b) : key[min(max(bi, 0), N - 1)];
        }
        for (int k = 0; k < nb; k++) {
            const int i = __builtin_amdgcn_readlane(bi, k);
            const uint32_t clo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)bc, k);
            const uint32_t chi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(bc >> 32), k);
            const unsigned long long ci = ((unsigned long long)chi << 32) | clo;
            if (top + cmax < (1ull << 24)) {                 // (clients are below 256: MMBP_MAX_M)
                uint32_t bk = 0xFFFFFFFFu;               // smallest (load, client) among this lane's clients with room
#pragma unroll
                for (int r = 0; r < kClientsPerLane; r++) {
                    const int j = lane + r * kWave;
                    if (j < M && cn[r] < cap) bk = min(bk, ((uint32_t)ld[r] << 8) | (uint32_t)j);
                }
                const uint32_t wk = wave_min_u32(bk);
                if (wk == 0xFFFFFFFFu) continue;         // cannot happen: N <= M * cap leaves room somewhere
                const uint32_t wj = wk & 255u;
#pragma unroll
                for (int r = 0; r < kClientsPerLane; r++)
                    if ((uint32_t)(lane + r * kWave) == wj) { ld[r] += ci; cn[r] += 1; }
                top = max(top, (unsigned long long)(wk >> 8) + ci);
                if (lane == 0 && i >= 0 && i < N) asg[i] = (int32_t)wj;
                continue;
            }
            // this lane's best client: smallest (load, client) among its clients with room
            unsigned long long bl = ~0ull;
            uint32_t bj = 0xFFFFFFFFu;
#pragma unroll
            for (int r = 0; r < kClientsPerLane; r++) {
                const int j = lane + r * kWave;
                if (j < M && cn[r] < cap && ld[r] < bl) { bl = ld[r]; bj = (uint32_t)j; }   // ascending j: ties keep the lower client
            }
            // wave-wide lexicographic minimum of (load hi, load lo, client)
            const uint32_t mh = wave_min_u32((uint32_t)(bl >> 32));
            const uint32_t ml = wave_min_u32((uint32_t)(bl >> 32) == mh ? (uint32_t)bl : 0xFFFFFFFFu);
            const bool mine = bj != 0xFFFFFFFFu && (uint32_t)(bl >> 32) == mh && (uint32_t)bl == ml;
            const uint32_t wj = wave_min_u32(mine ? bj : 0xFFFFFFFFu);
            if (wj == 0xFFFFFFFFu) continue;             // cannot happen: N <= M * cap leaves room somewhere
#pragma unroll
            for (int r = 0; r < kClientsPerLane; r++)
                if ((uint32_t)(lane + r * kWave) == wj) { ld[r] += ci; cn[r] += 1; }
            top = max(top, (((unsigned long long)mh << 32) | ml) + ci);
            if (lane == 0 && i >= 0 && i < N) asg[i] = (int32_t)wj;
        }
    }
#pragma unroll
    for (int r = 0; r < kClientsPerLane; r++) {
        const int j = lane + r * kWave;
        if (j < M) load_out[(size_t)s * M + j] = (int64_t)ld[r];
    }
    if (lane == 0) status_out[s] = MMBP_ST_OK;
}

}  // namespace

hipError_t launch_lpt_start(const void *cost, int dtype, int S, int N, int M, int cap, int32_t *assign_out,
                            int64_t *load_out, int32_t *order_out, int32_t *status_out, hipStream_t st)
{
    size_t P2 = 1;
    while ((long long)P2 < (long long)N) P2 <<= 1;
    const size_t bytes = P2 * sizeof(unsigned long long);
    hipError_t e;
#define MMBP_LPT_LAUNCH(T) \
    do { \
        if (bytes > 48 * 1024) { \
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(&lpt_start_kernel<T>), \
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)(MMBP_LPT_MAX_N * sizeof(unsigned long long))); \
            if (e != hipSuccess) return e; \
        } \
        lpt_start_kernel<T><<<dim3(S), dim3(kBlock), bytes, st>>>((const T *)cost, N, M, cap, assign_out, load_out, order_out, \
                                                                 status_out); \
    } while (0)
    if (dtype == MMBP_I32) MMBP_LPT_LAUNCH(int32_t);
    else MMBP_LPT_LAUNCH(int64_t);
#undef MMBP_LPT_LAUNCH
    return hipGetLastError();
}

}  // namespace mmbp
