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
// smallest absolute difference |y - x|, y = cu of the column, x = cu of the row - (l_a - l_b).
// With d = y - x taken modulo 2^32, the smallest d is the distance to the nearest column at or
// above x and the negated largest d the distance to the nearest column below x, so a candidate
// costs one v_sub_u32 plus half a v_min3_u32 and half a v_max3_u32, all full-rate VALU
// (v_sad_u32 would fuse them but issues at quarter rate).  Each unordered client pair is evaluated once; the client with the largest load
// ("critical") is always the column side, so the per-row minima against it are known for every
// other job.  They resolve the lowest-id tie-break exactly: an improving swap must involve the
// critical client, the jobs that take part in a best swap are read off the row minima, and only
// the few pairs that can carry the lowest id are re-examined.
//
// Exactness: all loads stay at or below the initial makespan T0; with T0 + 2*max T_i < 2^29 every
// quantity above is exact in 32 bits: x lies in (2^29, 3*2^29), a real |y - x| is below 2^29, a
// wrapped difference is above 7*2^29, and an empty column (cu = 6*2^29) gives d in (3*2^29, 5*2^29),
// which can win neither the minimum nor (negated) the maximum against a real column.  Scenarios
// that do not satisfy the bound stay pending for the 64-bit kernel.
#include "mmbp_dev.hpp"
#include "ls_tile.hpp"

namespace mmbp {
namespace {

#ifndef MMBP_LDS_CHUNK
#define MMBP_LDS_CHUNK 128
#endif
#ifndef MMBP_LDS_WPE
#define MMBP_LDS_WPE 4
#endif
constexpr int kChunk = MMBP_LDS_CHUNK;         // columns per task
constexpr size_t kLdsLimit = 64 * 1024;

struct Ctrl {
    unsigned long long evals;
    unsigned long long pairs_per_scan, pairs_before;
    unsigned long long wsum[16];
    unsigned long long wmax[16];
    long long T0;
    uint32_t vswap, vmove;
    int nfeas, P, rebuild;
    uint32_t top_v[3];            // three largest loads and their clients, published by wave 0
    int top_j[3];
    int passes, status, stop, iters;
    int bad_cost, bad_assign;
};

struct Lds {
    uint32_t *cu, *rowkey;   // rowkey[p]: best swap makespan of the job at p against the critical client
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

// Per-client counts, layout starts and loads as seen by one wave.  With M <= 64 they sit one per
// lane and are fetched with v_readlane (no LDS round trip in the task loop); otherwise they are
// read from LDS.
template <bool SMALLM>
struct Clients {
    const Lds *l;
    int maxn, maxp;               // clamps: a count never exceeds N, a start never exceeds the padded size
    uint32_t vcnt, vstart, vload;
    __device__ __forceinline__ void refresh(int M, int lane)
    {
        if (SMALLM) {
            vcnt = lane < M ? (uint32_t)l->cnt[lane] : 0u;
            vstart = lane < M ? (uint32_t)l->gstart[lane] : 0u;
            vload = lane < M ? (uint32_t)l->load[lane] : 0u;
        }
    }
    __device__ __forceinline__ int cnt(int g) const
    {
        const int v = SMALLM ? __builtin_amdgcn_readlane((int)vcnt, g) : __builtin_amdgcn_readfirstlane(l->cnt[g]);
        return min(max(v, 0), maxn);
    }
    __device__ __forceinline__ int start(int g) const
    {
        const int v = SMALLM ? __builtin_amdgcn_readlane((int)vstart, g) : __builtin_amdgcn_readfirstlane(l->gstart[g]);
        return min(max(v, 0), maxp) & ~63;
    }
    __device__ __forceinline__ uint32_t load(int g) const
    {
        return (uint32_t)(SMALLM ? __builtin_amdgcn_readlane((int)vload, g)
                                 : __builtin_amdgcn_readfirstlane((int)(uint32_t)l->load[g]));
    }
};

// three largest loads with their clients for M <= 64 (one load per lane): every lane ranks its
// load against all others (ties: lower client first), the lanes of rank 0, 1, 2 are read back
__device__ __forceinline__ Top3 wave_top3_small(uint32_t vload, int M, int lane)
{
    int rank = 0;
    for (int i = 0; i < M; i++) {
        const uint32_t li = (uint32_t)__builtin_amdgcn_readlane((int)vload, i);
        rank += (li > vload || (li == vload && i < lane)) ? 1 : 0;
    }
    Top3 t;
#pragma unroll
    for (int r = 0; r < 3; r++) {
        const unsigned long long m = __ballot(lane < M && rank == r);
        if (m) {
            const int j = __builtin_ctzll(m);
            t.j[r] = j;
            t.v[r] = (uint32_t)__builtin_amdgcn_readlane((int)vload, j);
        } else {
            t.j[r] = -1;
            t.v[r] = 0u;
        }
    }
    return t;
}

// One row unit (R row segments of client g starting at rowbase) against the column chunks whose
// flattened task index falls in [lo, hi); `first` is the task index of the unit's first chunk.
// Column clients of g: the non-empty clients after g except the critical one, then the critical
// one; each is cut into chunks of kChunk columns.  The best makespan of a row against the
// critical client is min-combined into rowkey (its chunks may run on different waves).
template <int R, bool SMALLM>
__device__ __forceinline__ void row_unit(const Lds &l, const Clients<SMALLM> &cl, const Top3 &top, int M, int astar,
                                         int g, uint32_t la, int rowbase, int lane, int first, int lo, int hi,
                                         uint32_t &sbest)
{
    uint32_t rowx[R];
#pragma unroll
    for (int r = 0; r < R; r++) rowx[r] = l.cu[rowbase + 64 * r + lane];
    int idx = first;
    for (int bb = g + 1; bb <= M; bb++) {
        const int b = (bb == M) ? astar : bb;
        if (bb < M && b == astar) continue;
        const int nb = cl.cnt(b);
        if (nb == 0) continue;
        const int nch = (nb + kChunk - 1) / kChunk;
        if (idx + nch <= lo) { idx += nch; continue; }
        if (idx >= hi) break;
        const uint32_t lb = cl.load(b);
        const int cbase = cl.start(b);
        const int cend = min(cbase + ((nb + 7) & ~7), cl.maxp);
        const uint32_t oth = others_max(top, g, b);
        const uint32_t lsum = la + lb;
        uint32_t x[R];
#pragma unroll
        for (int r = 0; r < R; r++) x[r] = rowx[r] - (la - lb);
        for (int ch = 0; ch < nch; ch++, idx++) {
            if (idx < lo) continue;
            if (idx >= hi) break;
            const int c0 = cbase + ch * kChunk;
            const int c1 = min(c0 + kChunk, cend);
            if (c1 <= c0) continue;
            uint32_t key[R];
            tile_columns<R>(l.cu, x, c0, c1, key);
#pragma unroll
            for (int r = 0; r < R; r++) {
                const uint32_t v = rowx[r] != kPad ? swap_value(key[r], lsum, oth) : kInf;
                sbest = min(sbest, v);
                if (b == astar && v != kInf) atomicMin(&l.rowkey[rowbase + 64 * r + lane], v);
            }
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
            const int ns = min((n + 63) >> 6, (N + 64 * M - pos) >> 6);
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
    for (int p = tid; p < P; p += BLOCK) { l.cu[p] = kPad; l.job[p] = kNoJob; l.rowkey[p] = kInf; }
    __syncthreads();
    for (int i = tid; i < N; i += BLOCK) {
        const int a = asg[i];
        const int p = l.gstart[a] + atomicAdd(&l.fillc[a], 1);
        l.cu[p] = 2u * (uint32_t)c[i] + kBias;
        l.job[p] = (uint16_t)i;
    }
    __syncthreads();
}

template <typename CostT, int BLOCK, bool SMALLM>
__global__ __launch_bounds__(BLOCK, MMBP_LDS_WPE) void ls_lds_kernel(
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
        ctrl->stop = 0; ctrl->evals = 0; ctrl->rebuild = 0; ctrl->pairs_before = 0;
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
        // exact 32-bit narrowing needs T0 + 2*max cost < 2^29
        if ((unsigned long long)ctrl->T0 + 2ull * cmax >= (unsigned long long)kNarrowLimit) {
            if (tid == 0) status_out[s] = kPending;
            return;
        }
    }
    build_layout<CostT, BLOCK>(l, c, asg, N, M, cap);

    // loads stay below 2^29 on this path: their low words are used
    auto load32 = [&](int g) -> uint32_t { return (uint32_t)l.load[g]; };
    Clients<SMALLM> cl;
    cl.l = &l;
    cl.maxn = N;
    cl.maxp = N + 64 * M;
    const int Pmax = N + 64 * M;

    // Opens a pass (wave 0 only, all 64 lanes): pass accounting and the three largest loads for
    // everybody.  Termination by construction: every loop of a pass is bounded by N, M and the
    // padded size, every barrier is reached under conditions read from LDS after a barrier, and
    // the pass loop itself is capped.
    auto open_pass = [&]() {
        __builtin_amdgcn_wave_barrier();   // lanes of a wave run in lockstep: lane 0's updates are complete
        if (lane == 0) {
            ctrl->iters += 1;
            if ((long long)ctrl->iters > (long long)max_passes + 1) { ctrl->status = MMBP_ST_INTERNAL; ctrl->stop = 1; }
            else if (ctrl->stop) { }
            else if (ctrl->passes == max_passes) { ctrl->status = MMBP_ST_TRUNCATED; ctrl->stop = 1; }
            else ctrl->evals += (unsigned long long)N * (unsigned long long)(M - 1) + ctrl->pairs_per_scan;
            ctrl->vswap = kInf; ctrl->vmove = kInf;
        }
        const Top3 t = SMALLM ? wave_top3_small(lane < M ? (uint32_t)l.load[lane] : 0u, M, lane)
                              : wave_top3(l.load, M, lane);
        if (lane == 0) {
            for (int r = 0; r < 3; r++) { ctrl->top_v[r] = t.v[r]; ctrl->top_j[r] = t.j[r]; }
        }
    };
    if (tid == 0) ctrl->iters = 0;
    if (wave == 0) open_pass();        // pairs_per_scan was set by build_layout (barrier inside)

    // ---------------- pass loop ----------------
    for (;;) {
        __syncthreads();                                 // B0: layout, loads, top-3 and flags are published
        if (ctrl->stop) break;
        if (ctrl->rebuild) {                             // a move was applied: regroup the jobs
            build_layout<CostT, BLOCK>(l, c, asg, N, M, cap);
            if (tid == 0) {                              // (after the last barrier of build_layout: nobody
                ctrl->rebuild = 0;                       //  reads the flag before the next B0)
                ctrl->evals -= ctrl->pairs_before;       // the pair count of the scan that starts now
                ctrl->evals += ctrl->pairs_per_scan;
            }
        }

        const int P = min(ctrl->P, Pmax) & ~63;
        const int nseg = P >> 6;
        const int nfeas = min(ctrl->nfeas, M);
        cl.refresh(M, lane);
        Top3 top;
        for (int r = 0; r < 3; r++) {
            top.v[r] = uniu(ctrl->top_v[r]);
            top.j[r] = uni(ctrl->top_j[r]);
        }
        const uint32_t T = top.v[0];
        const int astar = min(max(top.j[0], 0), M - 1);

        // ---- moves: value only ----
        uint32_t mbest = kInf;
        if (nfeas > 0) {
            for (int seg = wave; seg < nseg; seg += kWaves) {
                const int g = l.seg_grp[seg];
                const uint32_t x = l.cu[seg * 64 + lane];
                const uint32_t ci = (x - kBias) >> 1;
                const uint32_t la = load32(g);
                uint32_t m = kInf;
                for (int q = 0; q < nfeas; q++) {
                    const int b = l.feas[q];
                    if (b == g) continue;
                    const uint32_t v = max(max(la - ci, load32(b) + ci), others_max(top, g, b));
                    m = min(m, v);
                }
                if (x != kPad) mbest = min(mbest, m);
            }
        }

        // ---- swaps: value only.  Every unordered client pair once, the critical client always as
        // columns.  Tasks (row unit, column chunk) are numbered in row-major order and each wave
        // takes a contiguous range, so consecutive tasks of a wave reuse the rows in registers. ----
        uint32_t sbest = kInf;
        {
            const int nstar = cl.cnt(astar);
            const int chstar = (nstar + kChunk - 1) / kChunk;
            int ntask = 0, chafter = 0;                    // chunks of the non-empty, non-critical clients after g
            for (int g = M - 1; g >= 0; g--) {
                const int ng = cl.cnt(g);
                if (ng == 0 || g == astar) continue;
                ntask += ((((ng + 63) >> 6) + kRMax - 1) / kRMax) * (chafter + chstar);
                chafter += (ng + kChunk - 1) / kChunk;
            }
            const int lo = (int)(((long long)ntask * wave) / kWaves);
            const int hi = (int)(((long long)ntask * (wave + 1)) / kWaves);
            int base = 0;
            for (int g = 0; g < M && base < hi; g++) {
                const int ng = cl.cnt(g);
                if (ng == 0 || g == astar) continue;
                chafter -= (ng + kChunk - 1) / kChunk;
                const int ncol = chafter + chstar;
                const int gbase = cl.start(g);
                const int gseg = min((ng + 63) >> 6, (cl.maxp - gbase) >> 6);
                const uint32_t la = cl.load(g);
                for (int blk = 0; blk < gseg; blk += kRMax, base += ncol) {
                    if (base + ncol <= lo || base >= hi) continue;
                    const int rowbase = gbase + blk * 64;
                    switch (min(kRMax, gseg - blk)) {
                    case 1: row_unit<1, SMALLM>(l, cl, top, M, astar, g, la, rowbase, lane, base, lo, hi, sbest); break;
                    case 2: row_unit<2, SMALLM>(l, cl, top, M, astar, g, la, rowbase, lane, base, lo, hi, sbest); break;
                    case 3: row_unit<3, SMALLM>(l, cl, top, M, astar, g, la, rowbase, lane, base, lo, hi, sbest); break;
                    default: row_unit<4, SMALLM>(l, cl, top, M, astar, g, la, rowbase, lane, base, lo, hi, sbest); break;
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
        __syncthreads();                                 // B1: all candidate values are in
        if (wave != 0) continue;                         // selection, apply and the next pass opening: wave 0

        const uint32_t Vm = ctrl->vmove, Vs = ctrl->vswap;
        const uint32_t V = min(Vm, Vs);
        if (V >= T) {                                    // local optimum (status stays OK)
            if (lane == 0) ctrl->stop = 1;
            continue;
        }
        if (Vm <= Vs) {
            // ---- a move wins (move ids are below swap ids): lowest id among moves of value V ----
            unsigned long long best = ~0ull;
            for (int seg = 0; seg < nseg; seg++) {
                const int g = l.seg_grp[seg];
                const int p = seg * 64 + lane;
                const uint32_t x = l.cu[p];
                const uint32_t ci = (x - kBias) >> 1;
                const uint32_t la = load32(g);
                const uint32_t jb = l.job[p];
                for (int q = 0; q < nfeas; q++) {
                    const int b = l.feas[q];
                    if (b == g) continue;
                    const uint32_t v = max(max(la - ci, load32(b) + ci), others_max(top, g, b));
                    if (x != kPad && v == V) {
                        const unsigned long long id = (unsigned long long)jb * (unsigned long long)M + (unsigned long long)b;
                        best = min(best, (id << 32) | (unsigned long long)p);
                    }
                }
            }
            best = wave_min_u64(best);
            if (lane == 0) {
                const uint32_t id = (uint32_t)(best >> 32);
                const int p = (int)(uint32_t)best;
                const int i = (int)(id / (uint32_t)M), b = (int)(id % (uint32_t)M);
                if (best == ~0ull || i >= N || p >= P) {
                    ctrl->status = MMBP_ST_INTERNAL;     // cannot happen: the best move was found above
                    ctrl->stop = 1;
                } else {
                    const int a = l.seg_grp[p >> 6];
                    const long long ci = (long long)((l.cu[p] - kBias) >> 1);
                    l.load[a] -= ci; l.load[b] += ci;
                    l.cnt[a] -= 1; l.cnt[b] += 1;
                    asg[i] = b;
                    if (applied_log) applied_log[(size_t)s * max_passes + ctrl->passes] = (uint64_t)id;
                    ctrl->passes += 1;
                    ctrl->rebuild = 1;
                    ctrl->pairs_before = ctrl->pairs_per_scan;
                }
            }
            open_pass();
            continue;
        }

        // ---- a swap wins: lowest (min(i,k), max(i,k)) among swaps of value V.  An improving swap
        // involves the critical client, so every best swap pairs a critical job with a job whose
        // row minimum against the critical client equals V. ----
        const uint32_t lstar = load32(astar);
        const int sbase = min(max(l.gstart[astar], 0), P), scnt = min(max(l.cnt[astar], 0), P - sbase);
        const int send = sbase + scnt;
        // A: flagged jobs (non-critical side of a best swap), k0 = the lowest of them.  rowkey goes
        // back to "none" for the next pass while it is read.
        int nF = 0;
        unsigned long long k0 = ~0ull;
        for (int p0 = 0; p0 < P; p0 += kWave) {
            const int p = p0 + lane;
            const uint32_t v = l.rowkey[p];
            l.rowkey[p] = kInf;
            const bool flag = v == V;
            const unsigned long long m = __ballot(flag);
            if (flag) {
                l.list[nF + __popcll(m & ((1ull << lane) - 1ull))] = (uint16_t)p;
                k0 = min(k0, ((unsigned long long)l.job[p] << 32) | (unsigned long long)p);
            }
            nF += __popcll(m);
        }
        k0 = wave_min_u64(k0);
        if (k0 == ~0ull) {                               // cannot happen: a best swap has a flagged job
            if (lane == 0) { ctrl->status = MMBP_ST_INTERNAL; ctrl->stop = 1; }
            continue;
        }
        const uint32_t k0job = (uint32_t)(k0 >> 32);
        const int k0pos = min((int)(uint32_t)k0, P - 1);
        // B: critical jobs with a lower index than k0 (only they can give a lower id than k0's swaps)
        int nE = 0;
        for (int p0 = sbase; p0 < send; p0 += kWave) {
            const int p = p0 + lane;
            const bool early = p < send && (uint32_t)l.job[p] < k0job;
            const unsigned long long m = __ballot(early);
            if (early) l.list[P - 1 - (nE + __popcll(m & ((1ull << lane) - 1ull)))] = (uint16_t)p;
            nE += __popcll(m);
        }
        __builtin_amdgcn_wave_barrier();                 // the lists are read by other lanes of this wave
        // C: pairs (early critical job e, flagged job f), id (job_e, job_f);
        // D: pairs (k0, later critical job),              id (k0, job).
        // Candidates are packed (i:16 | k:16 | pos_i:16 | pos_k:16); the smallest wins.
        unsigned long long best = ~0ull;
        {
            const int npair = nE * nF;
            for (int q = lane; q < npair; q += kWave) {
                const int e = q / nF, f = q - e * nF;
                const int pe = l.list[P - 1 - e], pf = l.list[f];
                const int g = l.seg_grp[pf >> 6];
                const uint32_t lg = load32(g);
                const uint32_t key = absdiff_u32(l.cu[pe], l.cu[pf] - (lg - lstar));
                if (swap_value(key, lg + lstar, others_max(top, g, astar)) == V)
                    best = min(best, ((unsigned long long)l.job[pe] << 48) | ((unsigned long long)l.job[pf] << 32) |
                                         ((unsigned long long)pe << 16) | (unsigned long long)pf);
            }
            const int g = l.seg_grp[k0pos >> 6];
            const uint32_t lg = load32(g);
            const uint32_t xk = l.cu[k0pos] - (lg - lstar);
            const uint32_t oth = others_max(top, g, astar);
            for (int p = sbase + lane; p < send; p += kWave) {
                const uint32_t jb = l.job[p];
                if (jb > k0job && swap_value(absdiff_u32(l.cu[p], xk), lg + lstar, oth) == V)
                    best = min(best, ((unsigned long long)k0job << 48) | ((unsigned long long)jb << 32) |
                                         ((unsigned long long)k0pos << 16) | (unsigned long long)p);
            }
        }
        best = wave_min_u64(best);
        if (lane == 0) {
            const unsigned long long pr = best;
            const uint32_t ji = (uint32_t)(pr >> 48), jk = (uint32_t)(pr >> 32) & 0xFFFFu;     // ji < jk
            const int pi = (int)((pr >> 16) & 0xFFFFu), pk = (int)(pr & 0xFFFFu);
            if (pr == ~0ull || ji >= (uint32_t)N || jk >= (uint32_t)N || pi >= P || pk >= P) {
                ctrl->status = MMBP_ST_INTERNAL;         // cannot happen: the best swap was found above
                ctrl->stop = 1;
            } else {
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
        }
        open_pass();
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

template <typename CostT, int BLOCK, bool SMALLM>
hipError_t launch_one(const void *cost, int S, int N, int M, int cap, int max_passes, int32_t *assign,
                      int64_t *load_out, int64_t *makespan_out, int32_t *passes_out, uint64_t *evals_out,
                      uint64_t *applied_log, int32_t *status_out, hipStream_t st)
{
    size_t bytes = lds_bytes(N, M);
#ifdef MMBP_LDS_MINBYTES
    if (bytes < (size_t)(MMBP_LDS_MINBYTES)) bytes = (size_t)(MMBP_LDS_MINBYTES);
#endif
    ls_lds_kernel<CostT, BLOCK, SMALLM><<<dim3(S), dim3(BLOCK), bytes, st>>>(
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
    // workgroup size by padded problem size: more waves shorten a pass when the workgroup is alone
    // on its CU at the tail of a batch
#ifdef MMBP_LDS_FORCE_BLOCK
    const int block = (MMBP_LDS_FORCE_BLOCK);
#else
    const int pmax = N + 64 * M;
    const int block = pmax <= 2048 ? 256 : 512;
#endif
#define MMBP_LDS_LAUNCH(T, B, SM) \
    launch_one<T, B, SM>(cost, S, N, M, cap, max_passes, assign, load_out, makespan_out, passes_out, evals_out, \
                         applied_log, status_out, st)
#define MMBP_LDS_PICK(T) \
    (block == 256 ? (M <= 64 ? MMBP_LDS_LAUNCH(T, 256, true) : MMBP_LDS_LAUNCH(T, 256, false)) \
     : block == 512 ? (M <= 64 ? MMBP_LDS_LAUNCH(T, 512, true) : MMBP_LDS_LAUNCH(T, 512, false)) \
                    : (M <= 64 ? MMBP_LDS_LAUNCH(T, 1024, true) : MMBP_LDS_LAUNCH(T, 1024, false)))
    if (dtype == MMBP_I32) return MMBP_LDS_PICK(int32_t);
    return MMBP_LDS_PICK(int64_t);
#undef MMBP_LDS_PICK
#undef MMBP_LDS_LAUNCH
}

}  // namespace mmbp
