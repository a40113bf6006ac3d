// Multi-workgroup MMBP local search for scenarios that do not fit the LDS of one workgroup
// (e.g. one scenario with N = 65536, M = 64).  Same model, candidates, ids and tie-break as the
// LDS-resident kernel (ls_lds.hip); the state lives in the caller's workspace and a pass is two
// launches on the caller's stream:
//   grid_eval_kernel    every workgroup takes tasks (row block of client X x column chunk of client
//                       Y, Y staged in LDS) from a table and min-combines the best makespan into
//                       the control block, and per non-critical job its best makespan against the
//                       critical client (global argmin = atomic min of values, ids resolved later);
//   grid_select_kernel  one workgroup: picks the lowest-id candidate of the best value exactly
//                       (see ls_lds.hip), applies it, and prepares the next pass (top-3 loads,
//                       task table with the critical client always on the column side).
// The host enqueues min(max_passes, kMaxPassLaunches) such pairs; once a scenario has stopped the
// remaining launches return at once.
#include "mmbp_dev.hpp"
#include "ls_tile.hpp"

namespace mmbp {
namespace {

constexpr int kEvalBlock = 256;          // 4 waves, each up to kRMax row segments of a task's row block
#ifndef MMBP_GRID_EVAL_BLOCKS
#define MMBP_GRID_EVAL_BLOCKS 2048
#endif
constexpr int kEvalGrid = MMBP_GRID_EVAL_BLOCKS;   // workgroups of the evaluation kernel (stride loop over tasks)
constexpr int kSelBlock = 1024;
constexpr int kSelWaves = kSelBlock / kWave;
constexpr int kColChunk = 1024;          // columns staged in LDS per task
constexpr int kRowBlockSegs = (kEvalBlock / kWave) * kRMax;   // 16 segments = 1024 rows per task
constexpr int kMaxPassLaunches = 4096;
constexpr uint32_t kNoJob32 = 0xFFFFFFFFu;

struct GCtrl {
    unsigned long long evals, pairs_per_scan, k0, pair, mv;
    uint32_t vswap, vmove;
    Top3 top;
    int P, nfeas, ntask, passes, status, stop, iters, prune;
};

struct GTask {
    uint32_t xy;        // X | Y << 8 | nseg << 16   (row client, column client, row segments)
    uint32_t xrow0;     // first row position
    uint32_t ycol0;     // first column position
    uint32_t yncols;    // columns (multiple of 8)
};

__host__ __device__ inline size_t up256(size_t x) { return (x + 255) / 256 * 256; }

struct GLayout {        // byte offsets inside one scenario's workspace slice
    size_t ctrl, load, cnt, gstart, feas, cu, job, rowkey, list, seg_grp, tasks, total;
    int pmax, tmax;
};

__host__ __device__ inline GLayout grid_layout(int N, int M)
{
    GLayout g;
    g.pmax = N + 64 * M;
    g.tmax = (g.pmax / 1024 + M) * (N / 1024 + M);
    size_t o = 0;
    g.ctrl = o; o += up256(sizeof(GCtrl));
    g.load = o; o += up256(8 * (size_t)M);
    g.cnt = o; o += up256(4 * (size_t)(M + 1));
    g.gstart = o; o += up256(4 * (size_t)(M + 1));
    g.feas = o; o += up256(4 * (size_t)(M + 1));
    g.cu = o; o += up256(4 * (size_t)g.pmax);
    g.job = o; o += up256(4 * (size_t)g.pmax);
    g.rowkey = o; o += up256(4 * (size_t)g.pmax);
    g.list = o; o += up256(4 * (size_t)g.pmax);
    g.seg_grp = o; o += up256((size_t)g.pmax / 64 + 1);
    g.tasks = o; o += up256(sizeof(GTask) * (size_t)g.tmax);
    g.total = o;
    return g;
}

struct GWs {
    GCtrl *ctrl;
    long long *load;
    int *cnt, *gstart, *feas;
    uint32_t *cu, *job, *rowkey, *list;
    uint8_t *seg_grp;
    GTask *tasks;
    int pmax, tmax;
};

__device__ inline GWs grid_ws(void *workspace, int s, int N, int M)
{
    const GLayout g = grid_layout(N, M);
    unsigned char *b = (unsigned char *)workspace + (size_t)s * g.total;
    GWs w;
    w.ctrl = (GCtrl *)(b + g.ctrl);
    w.load = (long long *)(b + g.load);
    w.cnt = (int *)(b + g.cnt);
    w.gstart = (int *)(b + g.gstart);
    w.feas = (int *)(b + g.feas);
    w.cu = (uint32_t *)(b + g.cu);
    w.job = (uint32_t *)(b + g.job);
    w.rowkey = (uint32_t *)(b + g.rowkey);
    w.list = (uint32_t *)(b + g.list);
    w.seg_grp = (uint8_t *)(b + g.seg_grp);
    w.tasks = (GTask *)(b + g.tasks);
    w.pmax = g.pmax;
    w.tmax = g.tmax;
    return w;
}

struct OutPtrs {
    int64_t *load_out, *makespan_out;
    int32_t *passes_out, *status_out;
    uint64_t *evals_out, *applied_log;
};

// ---- pieces of the one-workgroup kernels (kSelBlock threads, all call) ----

// group the jobs by client: layout starts, segment -> client map, feasible move targets, pair count
template <typename CostT>
__device__ void g_build_layout(const GWs &w, const CostT *__restrict__ c, const int32_t *asg, int N, int M, int cap,
                               int *s_cursor)
{
    const int tid = threadIdx.x;
    if (tid == 0) {
        int pos = 0, nf = 0;
        unsigned long long sq = 0;
        for (int g = 0; g < M; g++) {
            w.gstart[g] = pos;
            const int n = w.cnt[g];
            pos += min((n + 63) >> 6, (w.pmax - pos) >> 6) * 64;
            if (n < cap) w.feas[nf++] = g;
            sq += (unsigned long long)n * (unsigned long long)n;
        }
        w.gstart[M] = pos;
        w.ctrl->P = pos;
        w.ctrl->nfeas = nf;
        w.ctrl->pairs_per_scan = ((unsigned long long)N * (unsigned long long)N - sq) / 2ull;
    }
    for (int j = tid; j < M; j += kSelBlock) s_cursor[j] = 0;
    __syncthreads();
    const int P = min(w.ctrl->P, w.pmax);
    for (int g = 0; g < M; g++)                       // segment -> client
        for (int sg = (w.gstart[g] >> 6) + tid; sg < (w.gstart[g + 1] >> 6); sg += kSelBlock) w.seg_grp[sg] = (uint8_t)g;
    for (int p = tid; p < P; p += kSelBlock) { w.cu[p] = kPad; w.job[p] = kNoJob32; }
    __syncthreads();
    for (int i = tid; i < N; i += kSelBlock) {
        const int a = asg[i];
        const int p = w.gstart[a] + atomicAdd(&s_cursor[a], 1);
        if (p < P) { w.cu[p] = 2u * (uint32_t)c[i] + kBias; w.job[p] = (uint32_t)i; }
    }
    __syncthreads();
}

__device__ void g_finish(const GWs &w, const OutPtrs &o, int s, int M)
{
    const int tid = threadIdx.x;
    for (int j = tid; j < M; j += kSelBlock) o.load_out[(size_t)s * M + j] = w.load[j];
    if (tid == 0) {
        long long t = 0;
        for (int j = 0; j < M; j++) t = max(t, w.load[j]);
        o.makespan_out[s] = t;
        o.passes_out[s] = w.ctrl->passes;
        if (o.evals_out) o.evals_out[s] = w.ctrl->evals;
        o.status_out[s] = w.ctrl->status;
        w.ctrl->stop = 1;
    }
}

// Opens a pass: accounting, top-3, reset of the row minima, task table.  Returns false (after
// writing the outputs) when the scenario stops here.
__device__ bool g_prep_pass(const GWs &w, const OutPtrs &o, int s, int N, int M, int max_passes, bool last_launch,
                            int *s_ntask)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    GCtrl *ctrl = w.ctrl;
    if (wave == 0) {
        if (lane == 0) {
            ctrl->iters += 1;
            if ((long long)ctrl->iters > (long long)max_passes + 1) { ctrl->status = MMBP_ST_INTERNAL; ctrl->stop = 1; }
            else if (ctrl->stop) { }
            else if (ctrl->passes == max_passes || last_launch) { ctrl->status = MMBP_ST_TRUNCATED; ctrl->stop = 1; }
            else ctrl->evals += (unsigned long long)N * (unsigned long long)(M - 1) + ctrl->pairs_per_scan;
            ctrl->vswap = kInf; ctrl->vmove = kInf;
            ctrl->k0 = ~0ull; ctrl->pair = ~0ull; ctrl->mv = ~0ull;
            *s_ntask = 0;
        }
        const Top3 t = wave_top3(w.load, M, lane);
        if (lane == 0) ctrl->top = t;
    }
    __syncthreads();
    if (ctrl->stop) { g_finish(w, o, s, M); return false; }
    const int P = min(ctrl->P, w.pmax);
    for (int p = tid; p < P; p += kSelBlock) w.rowkey[p] = kInf;
    // task table: every unordered pair of non-empty clients once, the critical client as columns
    const int astar = min(max(ctrl->top.j0, 0), M - 1);
    for (int q = tid; q < M * M; q += kSelBlock) {
        const int g = q / M, b = q - g * M;
        if (g >= b) continue;
        if (ctrl->prune && g != astar && b != astar) continue;      // pruned scan: pairs with the critical client only
        const int X = (g == astar) ? b : g, Y = (g == astar) ? g : b;
        const int nx = w.cnt[X], ny = w.cnt[Y];
        if (nx <= 0 || ny <= 0) continue;
        const int segx = (nx + 63) >> 6;
        const int nrb = (segx + kRowBlockSegs - 1) / kRowBlockSegs;
        const int ncols = (ny + 7) & ~7;
        const int ncc = (ncols + kColChunk - 1) / kColChunk;
        const int base = atomicAdd(s_ntask, nrb * ncc);
        if (base + nrb * ncc > w.tmax) continue;          // cannot happen (tmax bounds the table)
        for (int rb = 0; rb < nrb; rb++)
            for (int cc = 0; cc < ncc; cc++) {
                GTask e;
                e.xy = (uint32_t)X | ((uint32_t)Y << 8) | ((uint32_t)min(kRowBlockSegs, segx - rb * kRowBlockSegs) << 16);
                e.xrow0 = (uint32_t)(w.gstart[X] + rb * kRowBlockSegs * 64);
                e.ycol0 = (uint32_t)(w.gstart[Y] + cc * kColChunk);
                e.yncols = (uint32_t)min(kColChunk, ncols - cc * kColChunk);
                w.tasks[base + rb * ncc + cc] = e;
            }
    }
    __syncthreads();
    if (tid == 0) ctrl->ntask = min(*s_ntask, w.tmax);
    return true;
}

// ---- kernel 0: validation, narrowing decision, layout, first pass preparation ----
template <typename CostT>
__global__ __launch_bounds__(kSelBlock) void grid_stage_kernel(const CostT *__restrict__ cost_all, int N, int M, int cap,
                                                               int max_passes, int prune, int32_t *assign_all,
                                                               OutPtrs o, void *workspace)
{
    const int s = blockIdx.x;
    const GWs w = grid_ws(workspace, s, N, M);
    GCtrl *ctrl = w.ctrl;
    const CostT *c = cost_all + (size_t)s * N;
    const int32_t *asg = assign_all + (size_t)s * N;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    __shared__ long long s_load[MMBP_MAX_M];
    __shared__ int s_cnt[MMBP_MAX_M];
    __shared__ unsigned long long s_wsum[kSelWaves], s_wmax[kSelWaves];
    __shared__ int s_bad_cost, s_bad_assign, s_ntask;
    __shared__ long long s_T0;

    for (int j = tid; j < M; j += kSelBlock) { s_load[j] = 0; s_cnt[j] = 0; }
    if (tid == 0) {
        s_bad_cost = 0; s_bad_assign = 0;
        ctrl->passes = 0; ctrl->status = MMBP_ST_OK; ctrl->stop = 0; ctrl->evals = 0; ctrl->iters = 0; ctrl->ntask = 0;
        ctrl->prune = prune;
    }
    __syncthreads();
    {
        unsigned long long part = 0, cmax = 0;
        int my_bad_cost = 0, my_bad_assign = 0;
        for (int i = tid; i < N; i += kSelBlock) {
            const long long ci = (long long)c[i];
            const int a = asg[i];
            const bool cok = !(ci < 0 || ci >= kCostSumLimit);
            const bool aok = !(a < 0 || a >= M);
            if (!cok) my_bad_cost = 1;
            if (!aok) my_bad_assign = 1;
            if (cok) { part = sat_add62(part, (unsigned long long)ci); cmax = max(cmax, (unsigned long long)ci); }
            if (aok) atomicAdd(&s_cnt[a], 1);
            if (aok && cok) atomicAdd((unsigned long long *)&s_load[a], (unsigned long long)ci);
        }
        for (int off = 32; off >= 1; off >>= 1) {
            part = sat_add62(part, __shfl_xor(part, off));
            cmax = max(cmax, (unsigned long long)__shfl_xor(cmax, off));
        }
        if (lane == 0) { s_wsum[wave] = part; s_wmax[wave] = cmax; }
        if (my_bad_cost) s_bad_cost = 1;
        if (my_bad_assign) s_bad_assign = 1;
    }
    __syncthreads();
    for (int j = tid; j < M; j += kSelBlock)
        if (s_cnt[j] > cap) s_bad_assign = 1;
    if (tid == 0) {
        long long t0 = 0;
        for (int j = 0; j < M; j++) t0 = max(t0, s_load[j]);
        s_T0 = t0;
    }
    __syncthreads();
    unsigned long long tot = 0, cmax = 0;
    for (int q = 0; q < kSelWaves; q++) { tot = sat_add62(tot, s_wsum[q]); cmax = max(cmax, s_wmax[q]); }
    const bool bad_cost = s_bad_cost || tot >= (unsigned long long)kCostSumLimit;
    if (bad_cost || s_bad_assign) {
        for (int j = tid; j < M; j += kSelBlock) o.load_out[(size_t)s * M + j] = 0;
        if (tid == 0) {
            o.makespan_out[s] = 0; o.passes_out[s] = 0;
            if (o.evals_out) o.evals_out[s] = 0;
            o.status_out[s] = bad_cost ? MMBP_ST_BAD_COST : MMBP_ST_BAD_ASSIGN;
            ctrl->stop = 1;
        }
        return;
    }
    if ((unsigned long long)s_T0 + 2ull * cmax >= (unsigned long long)kNarrowLimit) {   // 64-bit kernel's job
        if (tid == 0) { o.status_out[s] = kPending; ctrl->stop = 1; }
        return;
    }
    for (int j = tid; j < M; j += kSelBlock) { w.load[j] = s_load[j]; w.cnt[j] = s_cnt[j]; }
    __syncthreads();
    g_build_layout<CostT>(w, c, asg, N, M, cap, s_cnt /* reused as cursors */);
    g_prep_pass(w, o, s, N, M, max_passes, false, &s_ntask);
}

// ---- kernel 1: evaluation of all candidates of a pass ----
template <int R>
__device__ __forceinline__ void eval_rows(const GWs &w, const uint32_t *cols, int ncols, int rowbase, int lane, uint32_t lx,
                                          uint32_t ly, uint32_t oth, bool y_is_star, uint32_t &sbest)
{
    uint32_t rowx[R], x[R], key[R];
#pragma unroll
    for (int r = 0; r < R; r++) {
        rowx[r] = w.cu[rowbase + 64 * r + lane];
        x[r] = rowx[r] - (lx - ly);
    }
    tile_columns<R>(cols, x, 0, ncols, key);
#pragma unroll
    for (int r = 0; r < R; r++) {
        const uint32_t v = rowx[r] != kPad ? swap_value(key[r], lx + ly, oth) : kInf;
        sbest = min(sbest, v);
        if (y_is_star && v != kInf) atomicMin(&w.rowkey[rowbase + 64 * r + lane], v);
    }
}

__global__ __launch_bounds__(kEvalBlock) void grid_eval_kernel(int N, int M, void *workspace)
{
    const int s = blockIdx.y;
    const GWs w = grid_ws(workspace, s, N, M);
    GCtrl *ctrl = w.ctrl;
    if (ctrl->stop) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    __shared__ __align__(16) uint32_t cols[kColChunk];
    Top3 top;
    top.v0 = uniu(ctrl->top.v0); top.v1 = uniu(ctrl->top.v1); top.v2 = uniu(ctrl->top.v2);
    top.j0 = uni(ctrl->top.j0); top.j1 = uni(ctrl->top.j1); top.j2 = uni(ctrl->top.j2);
    const int astar = min(max(top.j0, 0), M - 1);
    const int ntask = min(ctrl->ntask, w.tmax);
    const int P = min(ctrl->P, w.pmax);
    uint32_t sbest = kInf, mbest = kInf;

    for (int t = blockIdx.x; t < ntask; t += gridDim.x) {
        const GTask e = w.tasks[t];
        const int X = (int)(e.xy & 0xFFu), Y = (int)((e.xy >> 8) & 0xFFu), nseg = min((int)(e.xy >> 16), kRowBlockSegs);
        const int ncols = min((int)e.yncols, kColChunk) & ~7;
        const int ycol0 = max(min((int)e.ycol0, w.pmax - ncols), 0);
        for (int i = tid; i < ncols; i += kEvalBlock) cols[i] = w.cu[ycol0 + i];
        __syncthreads();
        const int rowbase = (int)e.xrow0 + wave * kRMax * 64;
        int R = min(max(nseg - wave * kRMax, 0), kRMax);
        if (rowbase < 0 || rowbase + 64 * R > w.pmax) R = 0;      // cannot happen: rows lie inside the layout
        if (R > 0 && ncols > 0) {
            const uint32_t lx = (uint32_t)w.load[X], ly = (uint32_t)w.load[Y];
            const uint32_t oth = others_max(top, X, Y);
            const bool star = Y == astar;
            switch (R) {
            case 1: eval_rows<1>(w, cols, ncols, rowbase, lane, lx, ly, oth, star, sbest); break;
            case 2: eval_rows<2>(w, cols, ncols, rowbase, lane, lx, ly, oth, star, sbest); break;
            case 3: eval_rows<3>(w, cols, ncols, rowbase, lane, lx, ly, oth, star, sbest); break;
            default: eval_rows<4>(w, cols, ncols, rowbase, lane, lx, ly, oth, star, sbest); break;
            }
        }
        __syncthreads();
    }
    // moves: value only
    const int nfeas = min(ctrl->nfeas, M);
    if (nfeas > 0) {
        const int nseg = P >> 6;
        for (int seg = blockIdx.x * (kEvalBlock / kWave) + wave; seg < nseg; seg += gridDim.x * (kEvalBlock / kWave)) {
            const int g = w.seg_grp[seg];
            if (ctrl->prune && g != astar) continue;                 // an improving move leaves the critical client
            const uint32_t x = w.cu[seg * 64 + lane];
            const uint32_t ci = (x - kBias) >> 1;
            const uint32_t la = (uint32_t)w.load[g];
            uint32_t m = kInf;
            for (int q = 0; q < nfeas; q++) {
                const int b = w.feas[q];
                if (b == g) continue;
                m = min(m, max(max(la - ci, (uint32_t)w.load[b] + ci), others_max(top, g, b)));
            }
            if (x != kPad) mbest = min(mbest, m);
        }
    }
    mbest = wave_min_u32(mbest);
    sbest = wave_min_u32(sbest);
    if (lane == 0) {
        if (mbest != kInf) atomicMin(&ctrl->vmove, mbest);
        if (sbest != kInf) atomicMin(&ctrl->vswap, sbest);
    }
}

// ---- kernel 2: exact selection, apply, preparation of the next pass ----
template <typename CostT>
__global__ __launch_bounds__(kSelBlock) void grid_select_kernel(const CostT *__restrict__ cost_all, int N, int M, int cap,
                                                                int max_passes, int32_t *assign_all, OutPtrs o,
                                                                void *workspace, int last_launch)
{
    const int s = blockIdx.x;
    const GWs w = grid_ws(workspace, s, N, M);
    GCtrl *ctrl = w.ctrl;
    if (ctrl->stop) return;
    const CostT *c = cost_all + (size_t)s * N;
    int32_t *asg = assign_all + (size_t)s * N;
    const int tid = threadIdx.x, lane = tid & 63;
    __shared__ int s_cursor[MMBP_MAX_M];
    __shared__ int s_nE, s_nF, s_ntask, s_rebuild;
    __shared__ unsigned long long s_k0, s_best;

    Top3 top;
    top.v0 = uniu(ctrl->top.v0); top.v1 = uniu(ctrl->top.v1); top.v2 = uniu(ctrl->top.v2);
    top.j0 = uni(ctrl->top.j0); top.j1 = uni(ctrl->top.j1); top.j2 = uni(ctrl->top.j2);
    const uint32_t T = top.v0;
    const int astar = min(max(top.j0, 0), M - 1);
    const int P = min(ctrl->P, w.pmax);
    const int nfeas = min(ctrl->nfeas, M);
    const uint32_t Vm = ctrl->vmove, Vs = ctrl->vswap;
    const uint32_t V = min(Vm, Vs);
    if (tid == 0) { s_nE = 0; s_nF = 0; s_rebuild = 0; s_k0 = ~0ull; s_best = ~0ull; }
    __syncthreads();
    if (V >= T) {                                        // local optimum
        g_finish(w, o, s, M);
        return;
    }
    if (Vm <= Vs) {
        // a move wins: lowest id among the moves of value V
        unsigned long long best = ~0ull;
        for (int p = tid; p < P; p += kSelBlock) {
            const uint32_t x = w.cu[p];
            if (x == kPad) continue;
            const int g = w.seg_grp[p >> 6];
            const uint32_t ci = (x - kBias) >> 1;
            const uint32_t la = (uint32_t)w.load[g];
            const uint32_t jb = w.job[p];
            for (int q = 0; q < nfeas; q++) {
                const int b = w.feas[q];
                if (b == g) continue;
                const uint32_t v = max(max(la - ci, (uint32_t)w.load[b] + ci), others_max(top, g, b));
                if (v == V)
                    best = min(best, (((unsigned long long)jb * (unsigned long long)M + (unsigned long long)b) << 32) |
                                         (unsigned long long)p);
            }
        }
        best = wave_min_u64(best);
        if (lane == 0 && best != ~0ull) atomicMin(&s_best, best);
        __syncthreads();
        if (tid == 0) {
            const unsigned long long mv = s_best;
            const uint32_t id = (uint32_t)(mv >> 32);
            const int p = (int)(uint32_t)mv;
            const int i = (int)(id / (uint32_t)M), b = (int)(id % (uint32_t)M);
            if (mv == ~0ull || i >= N || p >= P) { ctrl->status = MMBP_ST_INTERNAL; ctrl->stop = 1; }
            else {
                const int a = w.seg_grp[p >> 6];
                const long long ci = (long long)((w.cu[p] - kBias) >> 1);
                w.load[a] -= ci; w.load[b] += ci;
                w.cnt[a] -= 1; w.cnt[b] += 1;
                asg[i] = b;
                if (o.applied_log) o.applied_log[(size_t)s * max_passes + ctrl->passes] = (uint64_t)id;
                ctrl->passes += 1;
                s_rebuild = 1;
            }
        }
        __syncthreads();
        if (s_rebuild) g_build_layout<CostT>(w, c, asg, N, M, cap, s_cursor);
    } else {
        // a swap wins: lowest (min(i,k), max(i,k)) among the swaps of value V (see ls_lds.hip)
        const uint32_t lstar = (uint32_t)w.load[astar];
        const int sbase = min(max(w.gstart[astar], 0), P), scnt = min(max(w.cnt[astar], 0), P - sbase);
        const int send = sbase + scnt, sslots = sbase + ((scnt + 63) & ~63);
        {
            unsigned long long k0 = ~0ull;
            for (int p = tid; p < P; p += kSelBlock) {
                if (p >= sbase && p < sslots) continue;
                if (w.rowkey[p] == V) {
                    const int idx = atomicAdd(&s_nF, 1);
                    w.list[idx] = (uint32_t)p;
                    k0 = min(k0, ((unsigned long long)w.job[p] << 32) | (unsigned long long)p);
                }
            }
            k0 = wave_min_u64(k0);
            if (lane == 0 && k0 != ~0ull) atomicMin(&s_k0, k0);
        }
        __syncthreads();
        if (s_k0 == ~0ull) {                             // cannot happen: a best swap has a flagged job
            if (tid == 0) ctrl->status = MMBP_ST_INTERNAL;
            __syncthreads();
            g_finish(w, o, s, M);
            return;
        }
        const uint32_t k0job = (uint32_t)(s_k0 >> 32);
        const int k0pos = min((int)(uint32_t)s_k0, P - 1);
        for (int p = sbase + tid; p < send; p += kSelBlock) {
            if (w.job[p] < k0job) {
                const int idx = atomicAdd(&s_nE, 1);
                w.list[P - 1 - idx] = (uint32_t)p;
            }
        }
        __syncthreads();
        {
            // pairs (early critical job, flagged job) and (k0, later critical job); the packed
            // candidate (i << 44 | k << 24, job indices below 2^20) keeps the lowest (i, k)
            const int nE = min(s_nE, scnt), nF = min(s_nF, P);
            unsigned long long best = ~0ull;
            const long long npair = (long long)nE * (long long)nF;
            for (long long q = tid; q < npair; q += kSelBlock) {
                const int e = (int)(q / nF), f = (int)(q - (long long)e * nF);
                const int pe = (int)w.list[P - 1 - e], pf = (int)w.list[f];
                const int g = w.seg_grp[pf >> 6];
                const uint32_t lg = (uint32_t)w.load[g];
                const uint32_t key = absdiff_u32(w.cu[pe], w.cu[pf] - (lg - lstar));
                if (swap_value(key, lg + lstar, others_max(top, g, astar)) == V)
                    best = min(best, ((unsigned long long)w.job[pe] << 44) | ((unsigned long long)w.job[pf] << 24));
            }
            const int g = w.seg_grp[k0pos >> 6];
            const uint32_t lg = (uint32_t)w.load[g];
            const uint32_t xk = w.cu[k0pos] - (lg - lstar);
            const uint32_t oth = others_max(top, g, astar);
            for (int p = sbase + tid; p < send; p += kSelBlock) {
                const uint32_t jb = w.job[p];
                if (jb > k0job && swap_value(absdiff_u32(w.cu[p], xk), lg + lstar, oth) == V)
                    best = min(best, ((unsigned long long)k0job << 44) | ((unsigned long long)jb << 24));
            }
            best = wave_min_u64(best);
            if (lane == 0 && best != ~0ull) atomicMin(&s_best, best);
        }
        __syncthreads();
        // the winning jobs (i < k); their positions are looked up
        const unsigned long long pr = s_best;
        const uint32_t ji = (uint32_t)(pr >> 44), jk = (uint32_t)(pr >> 24) & 0xFFFFFu;
        if (tid == 0) { s_nE = -1; s_nF = -1; }
        __syncthreads();
        for (int p = tid; p < P; p += kSelBlock) {
            const uint32_t jb = w.job[p];
            if (jb == ji) s_nE = p;
            if (jb == jk) s_nF = p;
        }
        __syncthreads();
        if (tid == 0) {
            const int pi = s_nE, pk = s_nF;
            if (pr == ~0ull || ji >= (uint32_t)N || jk >= (uint32_t)N || pi < 0 || pk < 0) {
                ctrl->status = MMBP_ST_INTERNAL; ctrl->stop = 1;
            } else {
                const int ga = w.seg_grp[pi >> 6], gb = w.seg_grp[pk >> 6];
                const uint32_t xi = w.cu[pi], xk = w.cu[pk];
                const long long d = (long long)((xi - kBias) >> 1) - (long long)((xk - kBias) >> 1);
                w.load[ga] -= d; w.load[gb] += d;
                w.cu[pi] = xk; w.cu[pk] = xi;
                w.job[pi] = jk; w.job[pk] = ji;
                asg[ji] = gb; asg[jk] = ga;
                if (o.applied_log)
                    o.applied_log[(size_t)s * max_passes + ctrl->passes] =
                        (uint64_t)N * (uint64_t)M + (uint64_t)ji * (uint64_t)N + (uint64_t)jk;
                ctrl->passes += 1;
            }
        }
    }
    __syncthreads();
    g_prep_pass(w, o, s, N, M, max_passes, last_launch != 0, &s_ntask);
}

}  // namespace

size_t ls_grid_workspace_bytes(int S, int N, int M) { return (size_t)S * grid_layout(N, M).total; }

hipError_t launch_ls_grid(const void *cost, int dtype, int S, int N, int M, int cap, int max_passes, int prune,
                          int32_t *assign, int64_t *load_out, int64_t *makespan_out, int32_t *passes_out,
                          uint64_t *evals_out, uint64_t *applied_log, int32_t *status_out, void *workspace,
                          hipStream_t st)
{
    OutPtrs o{load_out, makespan_out, passes_out, status_out, evals_out, applied_log};
    if (dtype == MMBP_I32)
        grid_stage_kernel<int32_t><<<dim3(S), dim3(kSelBlock), 0, st>>>((const int32_t *)cost, N, M, cap, max_passes,
                                                                       prune, assign, o, workspace);
    else
        grid_stage_kernel<int64_t><<<dim3(S), dim3(kSelBlock), 0, st>>>((const int64_t *)cost, N, M, cap, max_passes,
                                                                       prune, assign, o, workspace);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int launches = max_passes < kMaxPassLaunches ? max_passes : kMaxPassLaunches;
    for (int i = 0; i < launches; i++) {
        grid_eval_kernel<<<dim3(kEvalGrid, S), dim3(kEvalBlock), 0, st>>>(N, M, workspace);
        const int last = (i == launches - 1 && launches < max_passes) ? 1 : 0;
        if (dtype == MMBP_I32)
            grid_select_kernel<int32_t><<<dim3(S), dim3(kSelBlock), 0, st>>>((const int32_t *)cost, N, M, cap, max_passes,
                                                                            assign, o, workspace, last);
        else
            grid_select_kernel<int64_t><<<dim3(S), dim3(kSelBlock), 0, st>>>((const int64_t *)cost, N, M, cap, max_passes,
                                                                            assign, o, workspace, last);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace mmbp
