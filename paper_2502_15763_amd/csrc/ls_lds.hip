// LDS-resident MMBP local search: one workgroup per scenario, the whole search (all passes) runs
// out of LDS and registers.
//
// Model (paper section "Offline requests scheduling & theoretical lower bound"): minimise
// max_j t_j, t_j = sum of the costs T_i assigned to client j.  A pass evaluates the makespan of
// every move and swap candidate and applies the smallest (makespan, id).
//
// Layout.  Jobs are kept grouped by client: client g owns the positions [gstart[g], gstart[g+1])
// (a multiple of 64, padded).  Per position: cu = 2*T_i + 2^30 and the job index.  For a swap of
// i (client a) with k (client b) the two changed loads are l_a - d and l_b + d, d = T_i - T_k, and
//     2 * max(l_a - d, l_b + d) = (l_a + l_b) + |(2 T_k + 2^30) - (2 T_i + 2^30 - (l_a - l_b))| .
// Inside a tile (64*R rows of client a) x (columns of client b), l_a, l_b and the largest
// untouched load are uniform, so the candidate with the smallest makespan is the one with the
// smallest absolute difference: one v_sad_u32 per candidate and one v_min3_u32 per two
// candidates.  Each unordered client pair is evaluated once; the client with the largest load
// ("critical") is always the column side, so the per-row minima against it are known for every
// other job.  They resolve the lowest-id tie-break exactly: an improving swap must involve the
// critical client, the jobs that take part in a best swap are read off the row minima, and only
// the few pairs that can carry the lowest id are re-examined.
//
// Exactness: all loads stay below the initial makespan T0; with T0 + 2*max T_i < 2^30 every
// quantity above fits 32 bits without wrap.  Scenarios that do not satisfy this stay pending for
// the 64-bit kernel.
#include "mmbp_dev.hpp"

namespace mmbp {
namespace {

constexpr uint32_t kBias = 1u << 30;
constexpr uint32_t kPad = 0xFFFFFFFFu;
constexpr uint32_t kKeyLimit = 1u << 30;      // every real key is below this
constexpr uint32_t kInf = 0xFFFFFFFFu;
constexpr uint16_t kNoJob = 0xFFFFu;
constexpr int kRMax = 4;                       // row segments (of 64 positions) per tile
constexpr size_t kLdsLimit = 64 * 1024;

struct Ctrl {
    unsigned long long k0;        // min (job << 32 | pos) over flagged non-critical jobs
    unsigned long long pair;      // min (job_e << 32 | job_f) over re-examined pairs
    unsigned long long mv;        // min (move id << 32 | pos)
    unsigned long long evals;
    unsigned long long pairs_per_scan;
    unsigned long long wsum[16];
    unsigned long long wmax[16];
    long long T0;
    uint32_t vswap, vmove, partner;
    int nE, nF, nfeas, P;
    int passes, status, stop;
    int bad_cost, bad_assign;
    int pos_i, pos_k;
};

struct Lds {
    uint32_t *cu, *rowkey;
    uint16_t *job, *list;
    long long *load;
    int *cnt, *gstart, *fillc, *feas;
    uint8_t *seg_grp;
    Ctrl *ctrl;
};

__host__ __device__ inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

__host__ __device__ inline size_t lds_bytes(int N, int M)
{
    const size_t P = (size_t)N + 64u * (size_t)M;
    size_t b = 0;
    b += 4 * P;                       // cu
    b += 4 * P;                       // rowkey
    b += 2 * P;                       // job
    b += 2 * P;                       // list
    b = align_up(b, 16);
    b += 8 * (size_t)M;               // load
    b += 4 * (size_t)(M + 1) * 4;     // cnt, gstart, fillc, feas
    b += align_up(P / 64 + 1, 16);    // seg_grp
    b = align_up(b, 16);
    b += sizeof(Ctrl);
    return b;
}

__device__ inline Lds carve(unsigned char *base, int N, int M)
{
    const size_t P = (size_t)N + 64u * (size_t)M;
    Lds l;
    size_t o = 0;
    l.cu = (uint32_t *)(base + o); o += 4 * P;
    l.rowkey = (uint32_t *)(base + o); o += 4 * P;
    l.job = (uint16_t *)(base + o); o += 2 * P;
    l.list = (uint16_t *)(base + o); o += 2 * P;
    o = align_up(o, 16);
    l.load = (long long *)(base + o); o += 8 * (size_t)M;
    l.cnt = (int *)(base + o); o += 4 * (size_t)(M + 1);
    l.gstart = (int *)(base + o); o += 4 * (size_t)(M + 1);
    l.fillc = (int *)(base + o); o += 4 * (size_t)(M + 1);
    l.feas = (int *)(base + o); o += 4 * (size_t)(M + 1);
    l.seg_grp = (uint8_t *)(base + o); o += align_up(P / 64 + 1, 16);
    o = align_up(o, 16);
    l.ctrl = (Ctrl *)(base + o);
    return l;
}

__device__ __forceinline__ uint32_t sad_u32(uint32_t a, uint32_t b)
{
    uint32_t d;
    asm("v_sad_u32 %0, %1, %2, 0" : "=v"(d) : "v"(a), "v"(b));
    return d;
}
__device__ __forceinline__ uint32_t min3_u32(uint32_t a, uint32_t b, uint32_t c)
{
    uint32_t d;
    asm("v_min3_u32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
    return d;
}

__device__ __forceinline__ unsigned long long sat_add62(unsigned long long a, unsigned long long b)
{
    unsigned long long r = a + b;
    return r >= (unsigned long long)kCostSumLimit ? (unsigned long long)kCostSumLimit : r;
}

__device__ __forceinline__ int uni(int x) { return __builtin_amdgcn_readfirstlane(x); }
__device__ __forceinline__ uint32_t uniu(uint32_t x) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)x); }

// three largest loads with their clients (lowest client index first among equal loads)
struct Top3 {
    uint32_t v[3];
    int j[3];
};

__device__ __forceinline__ Top3 wave_top3(const long long *load, int M, int lane)
{
    Top3 t;
    int ex0 = -1, ex1 = -1;
#pragma unroll
    for (int r = 0; r < 3; r++) {
        uint32_t bv = 0, bj = kInf;
        for (int j = lane; j < M; j += kWave) {
            if (j == ex0 || j == ex1) continue;
            uint32_t l = (uint32_t)load[j];
            if (bj == kInf || l > bv) { bv = l; bj = (uint32_t)j; }
        }
        uint32_t mv = wave_max_u32(bv);
        uint32_t mj = wave_min_u32((bv == mv) ? bj : kInf);
        t.v[r] = (mj == kInf) ? 0u : mv;
        t.j[r] = (int)mj;                       // -1 when fewer than r+1 clients
        if (r == 0) ex0 = (int)mj; else ex1 = (int)mj;
    }
    return t;
}

__device__ __forceinline__ uint32_t others_max(const Top3 &t, int a, int b)
{
    if (t.j[0] != a && t.j[0] != b) return t.v[0];
    if (t.j[1] != a && t.j[1] != b) return t.v[1];
    return t.v[2];
}

// makespan of a swap candidate from its key (absolute difference), the two loads and the largest
// untouched load
__device__ __forceinline__ uint32_t swap_value(uint32_t key, uint32_t lsum, uint32_t others)
{
    return key < kKeyLimit ? max(others, (lsum + key) >> 1) : kInf;
}

// Tile: R row segments starting at rowbase against the columns [c0, c1) ((c1 - c0) % 8 == 0).
// acc[r] = min over the columns of |cu[col] - (cu[row] - delta)|.
template <int R>
__device__ __forceinline__ void swap_tile(const uint32_t *cu, int rowbase, int lane, uint32_t delta, int c0, int c1,
                                          uint32_t (&acc)[kRMax], uint32_t (&rowx)[kRMax])
{
    uint32_t g[R];
#pragma unroll
    for (int r = 0; r < R; r++) {
        rowx[r] = cu[rowbase + 64 * r + lane];
        g[r] = rowx[r] - delta;
        acc[r] = kInf;
    }
    const uint4 *col = reinterpret_cast<const uint4 *>(cu + c0);
    const int n4 = (c1 - c0) >> 2;
    for (int k = 0; k < n4; k += 2) {
        const uint4 u = col[k];
        const uint4 w = col[k + 1];
#pragma unroll
        for (int r = 0; r < R; r++) {
            acc[r] = min3_u32(acc[r], sad_u32(u.x, g[r]), sad_u32(u.y, g[r]));
            acc[r] = min3_u32(acc[r], sad_u32(u.z, g[r]), sad_u32(u.w, g[r]));
            acc[r] = min3_u32(acc[r], sad_u32(w.x, g[r]), sad_u32(w.y, g[r]));
            acc[r] = min3_u32(acc[r], sad_u32(w.z, g[r]), sad_u32(w.w, g[r]));
        }
    }
}

template <typename CostT, int BLOCK>
__device__ void build_layout(const Lds &l, const CostT *__restrict__ c, const int32_t *asg, int N, int M, int cap)
{
    const int tid = threadIdx.x;
    if (tid == 0) {
        int pos = 0, nf = 0;
        unsigned long long sq = 0;
        for (int g = 0; g < M; g++) {
            l.gstart[g] = pos;
            const int n = l.cnt[g];
            const int ns = (n + 63) >> 6;
            for (int q = 0; q < ns; q++) l.seg_grp[(pos >> 6) + q] = (uint8_t)g;
            pos += ns * 64;
            if (n < cap) l.feas[nf++] = g;
            sq += (unsigned long long)n * (unsigned long long)n;
        }
        l.gstart[M] = pos;
        l.ctrl->P = pos;
        l.ctrl->nfeas = nf;
        l.ctrl->pairs_per_scan = ((unsigned long long)N * (unsigned long long)N - sq) / 2ull;
    }
    for (int j = tid; j < M; j += BLOCK) l.fillc[j] = 0;
    __syncthreads();
    const int P = l.ctrl->P;
    for (int p = tid; p < P; p += BLOCK) { l.cu[p] = kPad; l.job[p] = kNoJob; }
    __syncthreads();
    for (int i = tid; i < N; i += BLOCK) {
        const int a = asg[i];
        const int p = l.gstart[a] + atomicAdd(&l.fillc[a], 1);
        l.cu[p] = 2u * (uint32_t)c[i] + kBias;
        l.job[p] = (uint16_t)i;
    }
    __syncthreads();
}

template <typename CostT, int BLOCK>
__global__ __launch_bounds__(BLOCK) void ls_lds_kernel(
    const CostT *__restrict__ cost_all, int N, int M, int cap, int max_passes, int32_t *assign_all,
    int64_t *load_out, int64_t *makespan_out, int32_t *passes_out, uint64_t *evals_out,
    uint64_t *applied_log, int32_t *status_out)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const Lds l = carve(lds_raw, N, M);
    Ctrl *ctrl = l.ctrl;
    const int s = blockIdx.x;
    const CostT *c = cost_all + (size_t)s * N;
    int32_t *asg = assign_all + (size_t)s * N;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int kWaves = BLOCK / kWave;

    // ---------------- stage: validation, counts, loads ----------------
    for (int j = tid; j < M; j += BLOCK) { l.load[j] = 0; l.cnt[j] = 0; }
    if (tid == 0) {
        ctrl->bad_cost = 0; ctrl->bad_assign = 0; ctrl->passes = 0; ctrl->status = MMBP_ST_OK;
        ctrl->stop = 0; ctrl->evals = 0;
    }
    __syncthreads();
    {
        unsigned long long part = 0, cmax = 0;
        int my_bad_cost = 0, my_bad_assign = 0;
        for (int i = tid; i < N; i += BLOCK) {
            const long long ci = (long long)c[i];
            const int a = asg[i];
            const bool cok = !(ci < 0 || ci >= kCostSumLimit);
            const bool aok = !(a < 0 || a >= M);
            if (!cok) my_bad_cost = 1;
            if (!aok) my_bad_assign = 1;
            if (cok) { part = sat_add62(part, (unsigned long long)ci); cmax = max(cmax, (unsigned long long)ci); }
            if (aok) atomicAdd(&l.cnt[a], 1);
            if (aok && cok) atomicAdd((unsigned long long *)&l.load[a], (unsigned long long)ci);
        }
        for (int off = 32; off >= 1; off >>= 1) {
            part = sat_add62(part, __shfl_xor(part, off));
            cmax = max(cmax, (unsigned long long)__shfl_xor(cmax, off));
        }
        if (lane == 0) { ctrl->wsum[wave] = part; ctrl->wmax[wave] = cmax; }
        if (my_bad_cost) ctrl->bad_cost = 1;
        if (my_bad_assign) ctrl->bad_assign = 1;
    }
    __syncthreads();
    for (int j = tid; j < M; j += BLOCK)
        if (l.cnt[j] > cap) ctrl->bad_assign = 1;
    if (tid == 0) {
        long long t0 = 0;
        for (int j = 0; j < M; j++) t0 = max(t0, l.load[j]);
        ctrl->T0 = t0;
    }
    __syncthreads();
    {
        unsigned long long tot = 0, cmax = 0;
#pragma unroll
        for (int w = 0; w < kWaves; w++) { tot = sat_add62(tot, ctrl->wsum[w]); cmax = max(cmax, ctrl->wmax[w]); }
        const bool bad_cost = ctrl->bad_cost || tot >= (unsigned long long)kCostSumLimit;
        if (bad_cost || ctrl->bad_assign) {
            for (int j = tid; j < M; j += BLOCK) load_out[(size_t)s * M + j] = 0;
            if (tid == 0) {
                makespan_out[s] = 0; passes_out[s] = 0;
                if (evals_out) evals_out[s] = 0;
                status_out[s] = bad_cost ? MMBP_ST_BAD_COST : MMBP_ST_BAD_ASSIGN;
            }
            return;
        }
        // exact 32-bit narrowing needs T0 + 2*max cost < 2^30
        if ((unsigned long long)ctrl->T0 + 2ull * cmax >= (unsigned long long)kKeyLimit) {
            if (tid == 0) status_out[s] = kPending;
            return;
        }
    }
    build_layout<CostT, BLOCK>(l, c, asg, N, M, cap);

    const uint32_t *load32 = reinterpret_cast<const uint32_t *>(l.load);   // low words (loads < 2^30)

    // ---------------- pass loop ----------------
    for (;;) {
        if (tid == 0) {
            if (ctrl->passes == max_passes) { ctrl->status = MMBP_ST_TRUNCATED; ctrl->stop = 1; }
            else ctrl->evals += (unsigned long long)N * (unsigned long long)(M - 1) + ctrl->pairs_per_scan;
            ctrl->vswap = kInf; ctrl->vmove = kInf; ctrl->partner = kInf;
            ctrl->k0 = ~0ull; ctrl->pair = ~0ull; ctrl->mv = ~0ull;
            ctrl->nE = 0; ctrl->nF = 0;
        }
        __syncthreads();
        if (ctrl->stop) break;

        const int P = ctrl->P;
        const int nseg = P >> 6;
        const int nfeas = ctrl->nfeas;
        const Top3 top = wave_top3(l.load, M, lane);
        const uint32_t T = top.v[0];
        const int astar = top.j[0];

        // ---- moves: value only ----
        uint32_t mbest = kInf;
        if (nfeas > 0) {
            for (int seg = wave; seg < nseg; seg += kWaves) {
                const int g = l.seg_grp[seg];
                const uint32_t x = l.cu[seg * 64 + lane];
                const uint32_t ci = (x - kBias) >> 1;
                const uint32_t la = load32[2 * g];
                uint32_t m = kInf;
                for (int q = 0; q < nfeas; q++) {
                    const int b = l.feas[q];
                    if (b == g) continue;
                    const uint32_t v = max(max(la - ci, load32[2 * b] + ci), others_max(top, g, b));
                    m = min(m, v);
                }
                if (x != kPad) mbest = min(mbest, m);
            }
        }

        // ---- swaps: value only, every unordered client pair once, critical client as columns ----
        uint32_t sbest = kInf;
        {
            int tcount = 0;
            for (int g = 0; g < M; g++) {
                const int ng = l.cnt[g];
                if (g == astar || ng == 0) continue;
                const int gseg = (ng + 63) >> 6;
                const int gbase = l.gstart[g];
                const uint32_t la = load32[2 * g];
                for (int blk = 0; blk < gseg; blk += kRMax) {
                    const int R = min(kRMax, gseg - blk);
                    const int rowbase = gbase + blk * 64;
                    for (int bb = g + 1; bb <= M; bb++) {
                        const int b = (bb == M) ? astar : bb;
                        if (bb < M && b == astar) continue;
                        const int nb = l.cnt[b];
                        if (nb == 0) continue;
                        if ((tcount++ % kWaves) != wave) continue;
                        const uint32_t lb = load32[2 * b];
                        const int c0 = l.gstart[b];
                        const int c1 = c0 + ((nb + 7) & ~7);
                        uint32_t acc[kRMax], rowx[kRMax];
                        switch (R) {
                        case 1: swap_tile<1>(l.cu, rowbase, lane, la - lb, c0, c1, acc, rowx); break;
                        case 2: swap_tile<2>(l.cu, rowbase, lane, la - lb, c0, c1, acc, rowx); break;
                        case 3: swap_tile<3>(l.cu, rowbase, lane, la - lb, c0, c1, acc, rowx); break;
                        default: swap_tile<4>(l.cu, rowbase, lane, la - lb, c0, c1, acc, rowx); break;
                        }
                        const uint32_t oth = others_max(top, g, b);
                        const uint32_t lsum = la + lb;
                        for (int r = 0; r < R; r++) {
                            if (rowx[r] != kPad) sbest = min(sbest, swap_value(acc[r], lsum, oth));
                            if (b == astar) l.rowkey[rowbase + 64 * r + lane] = acc[r];
                        }
                    }
                }
            }
        }
        mbest = wave_min_u32(mbest);
        sbest = wave_min_u32(sbest);
        if (lane == 0) {
            if (mbest != kInf) atomicMin(&ctrl->vmove, mbest);
            if (sbest != kInf) atomicMin(&ctrl->vswap, sbest);
        }
        __syncthreads();

        const uint32_t Vm = ctrl->vmove, Vs = ctrl->vswap;
        const uint32_t V = min(Vm, Vs);
        if (V >= T) break;                               // local optimum (status stays OK)

        if (Vm <= Vs) {
            // ---- a move wins (move ids are below swap ids): lowest id among moves of value V ----
            unsigned long long best = ~0ull;
            for (int seg = wave; seg < nseg; seg += kWaves) {
                const int g = l.seg_grp[seg];
                const int p = seg * 64 + lane;
                const uint32_t x = l.cu[p];
                if (x == kPad) continue;
                const uint32_t ci = (x - kBias) >> 1;
                const uint32_t la = load32[2 * g];
                const uint32_t jb = l.job[p];
                for (int q = 0; q < nfeas; q++) {
                    const int b = l.feas[q];
                    if (b == g) continue;
                    const uint32_t v = max(max(la - ci, load32[2 * b] + ci), others_max(top, g, b));
                    if (v == V) {
                        const unsigned long long id = (unsigned long long)jb * (unsigned long long)M + (unsigned long long)b;
                        best = min(best, (id << 32) | (unsigned long long)p);
                    }
                }
            }
            best = wave_min_u64(best);
            if (lane == 0 && best != ~0ull) atomicMin(&ctrl->mv, best);
            __syncthreads();
            if (tid == 0) {
                const unsigned long long mvv = ctrl->mv;
                const uint32_t id = (uint32_t)(mvv >> 32);
                const int p = (int)(uint32_t)mvv;
                const int i = (int)(id / (uint32_t)M), b = (int)(id % (uint32_t)M);
                const int a = l.seg_grp[p >> 6];
                const long long ci = (long long)((l.cu[p] - kBias) >> 1);
                l.load[a] -= ci; l.load[b] += ci;
                l.cnt[a] -= 1; l.cnt[b] += 1;
                asg[i] = b;
                if (applied_log) applied_log[(size_t)s * max_passes + ctrl->passes] = (uint64_t)id;
                ctrl->passes += 1;
            }
            __syncthreads();
            build_layout<CostT, BLOCK>(l, c, asg, N, M, cap);
            continue;
        }

        // ---- a swap wins: lowest (min(i,k), max(i,k)) among swaps of value V ----
        const uint32_t lstar = load32[2 * astar];
        // A: non-critical jobs that take part in a best swap (from the row minima against the critical client)
        {
            unsigned long long k0 = ~0ull;
            for (int p = tid; p < P; p += BLOCK) {
                const int g = l.seg_grp[p >> 6];
                const uint32_t jb = l.job[p];
                if (g == astar || jb == kNoJob) continue;
                const uint32_t v = swap_value(l.rowkey[p], load32[2 * g] + lstar, others_max(top, g, astar));
                if (v == V) {
                    const int idx = atomicAdd(&ctrl->nF, 1);
                    l.list[idx] = (uint16_t)p;
                    k0 = min(k0, ((unsigned long long)jb << 32) | (unsigned long long)p);
                }
            }
            k0 = wave_min_u64(k0);
            if (lane == 0 && k0 != ~0ull) atomicMin(&ctrl->k0, k0);
        }
        __syncthreads();
        const uint32_t k0job = (uint32_t)(ctrl->k0 >> 32);
        const int k0pos = (int)(uint32_t)ctrl->k0;
        const int sbase = l.gstart[astar], send = sbase + l.cnt[astar];
        // B: critical-client jobs with a lower index than k0 (only they can give a lower id)
        for (int p = sbase + tid; p < send; p += BLOCK) {
            if ((uint32_t)l.job[p] < k0job) {
                const int idx = atomicAdd(&ctrl->nE, 1);
                l.list[P - 1 - idx] = (uint16_t)p;
            }
        }
        __syncthreads();
        const int nE = ctrl->nE, nF = ctrl->nF;
        if (nE > 0) {
            // C: pairs (early critical job, flagged job): waves over the former, lanes over the latter
            unsigned long long best = ~0ull;
            for (int e = wave; e < nE; e += kWaves) {
                const int pe = l.list[P - 1 - e];
                const uint32_t xe = l.cu[pe];
                const unsigned long long je = (unsigned long long)l.job[pe] << 32;
                for (int f = lane; f < nF; f += kWave) {
                    const int pf = l.list[f];
                    const int g = l.seg_grp[pf >> 6];
                    const uint32_t lg = load32[2 * g];
                    const uint32_t key = sad_u32(xe, l.cu[pf] - (lg - lstar));
                    if (swap_value(key, lg + lstar, others_max(top, g, astar)) == V)
                        best = min(best, je | (unsigned long long)l.job[pf]);
                }
            }
            best = wave_min_u64(best);
            if (lane == 0 && best != ~0ull) atomicMin(&ctrl->pair, best);
            __syncthreads();
        }
        unsigned long long pr = (nE > 0) ? ctrl->pair : ~0ull;
        if (pr == ~0ull) {
            // D: k0 is the lower index of the best swap; its partner is the lowest critical job paired with it
            const int g = l.seg_grp[k0pos >> 6];
            const uint32_t lg = load32[2 * g];
            const uint32_t gk = l.cu[k0pos] - (lg - lstar);
            const uint32_t oth = others_max(top, g, astar);
            uint32_t pj = kInf;
            for (int p = sbase + tid; p < send; p += BLOCK) {
                const uint32_t key = sad_u32(l.cu[p], gk);
                if (swap_value(key, lg + lstar, oth) == V) pj = min(pj, (uint32_t)l.job[p]);
            }
            pj = wave_min_u32(pj);
            if (lane == 0 && pj != kInf) atomicMin(&ctrl->partner, pj);
            __syncthreads();
            pr = ((unsigned long long)k0job << 32) | (unsigned long long)ctrl->partner;
        }
        const uint32_t ji = (uint32_t)(pr >> 32), jk = (uint32_t)pr;     // ji < jk
        // positions of the two jobs
        for (int p = tid; p < P; p += BLOCK) {
            const uint32_t jb = l.job[p];
            if (jb == ji) ctrl->pos_i = p;
            if (jb == jk) ctrl->pos_k = p;
        }
        __syncthreads();
        if (tid == 0) {
            const int pi = ctrl->pos_i, pk = ctrl->pos_k;
            const int ga = l.seg_grp[pi >> 6], gb = l.seg_grp[pk >> 6];
            const uint32_t xi = l.cu[pi], xk = l.cu[pk];
            const long long d = (long long)((xi - kBias) >> 1) - (long long)((xk - kBias) >> 1);
            l.load[ga] -= d; l.load[gb] += d;
            l.cu[pi] = xk; l.cu[pk] = xi;
            l.job[pi] = (uint16_t)jk; l.job[pk] = (uint16_t)ji;
            asg[ji] = gb; asg[jk] = ga;
            if (applied_log)
                applied_log[(size_t)s * max_passes + ctrl->passes] =
                    (uint64_t)N * (uint64_t)M + (uint64_t)ji * (uint64_t)N + (uint64_t)jk;
            ctrl->passes += 1;
        }
        // the barrier at the top of the next pass orders the update before its readers
    }

    // ---------------- write back ----------------
    __syncthreads();
    for (int j = tid; j < M; j += BLOCK) load_out[(size_t)s * M + j] = l.load[j];
    if (tid == 0) {
        long long t = 0;
        for (int j = 0; j < M; j++) t = max(t, l.load[j]);
        makespan_out[s] = t;
        passes_out[s] = ctrl->passes;
        if (evals_out) evals_out[s] = ctrl->evals;
        status_out[s] = ctrl->status;
    }
}

template <typename CostT, int BLOCK>
hipError_t launch_one(const void *cost, int S, int N, int M, int cap, int max_passes, int32_t *assign,
                      int64_t *load_out, int64_t *makespan_out, int32_t *passes_out, uint64_t *evals_out,
                      uint64_t *applied_log, int32_t *status_out, hipStream_t st)
{
    const size_t bytes = lds_bytes(N, M);
    ls_lds_kernel<CostT, BLOCK><<<dim3(S), dim3(BLOCK), bytes, st>>>(
        (const CostT *)cost, N, M, cap, max_passes, assign, load_out, makespan_out, passes_out, evals_out,
        applied_log, status_out);
    return hipGetLastError();
}

}  // namespace

bool ls_lds_fits(int N, int M) { return N < 65535 && lds_bytes(N, M) <= kLdsLimit; }

hipError_t launch_ls_lds(const void *cost, int dtype, int S, int N, int M, int cap, int max_passes,
                         int32_t *assign, int64_t *load_out, int64_t *makespan_out, int32_t *passes_out,
                         uint64_t *evals_out, uint64_t *applied_log, int32_t *status_out, hipStream_t st)
{
    const bool big = (N + 64 * M) > 2048;
#define MMBP_LDS_LAUNCH(T, B) \
    launch_one<T, B>(cost, S, N, M, cap, max_passes, assign, load_out, makespan_out, passes_out, evals_out, \
                     applied_log, status_out, st)
    if (dtype == MMBP_I32) return big ? MMBP_LDS_LAUNCH(int32_t, 512) : MMBP_LDS_LAUNCH(int32_t, 256);
    return big ? MMBP_LDS_LAUNCH(int64_t, 512) : MMBP_LDS_LAUNCH(int64_t, 256);
#undef MMBP_LDS_LAUNCH
}

}  // namespace mmbp
