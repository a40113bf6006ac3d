// Multi-workgroup MMBP local search for scenarios that do not fit the LDS of one workgroup
// (e.g. one scenario with N = 65536, M = 64).  Same model, candidates, ids and tie-break as the
// LDS-resident kernel (ls_lds.hip); the state lives in the caller's workspace and a pass is three
// launches on the caller's stream:
//   grid_eval_kernel    every workgroup takes tasks (row block of client X x column chunk of client
//                       Y, Y staged in LDS) from a table and min-combines the best makespan into
//                       the control block, and per non-critical job its best makespan against the
//                       critical client (global argmin = atomic min of values, ids resolved later);
//   grid_flag_kernel    many workgroups: when a swap wins, the flagged job of lowest index and the
//                       lowest partners of the four critical jobs of lowest index (one pass over
//                       the layout); resets the row minima buffer of the next pass;
//   grid_select_kernel  one workgroup: picks the lowest-id candidate of the best value exactly,
//                       applies it, and prepares the next pass (top-3 loads, task table with the
//                       critical client always on the column side).
// The host enqueues max_passes (at most kMaxPassLaunches; callers of larger limits that could run on
// one workgroup are routed there, others are refused) such triples (pairs for small layouts, which
// the selection workgroup scans itself); once a scenario has stopped the remaining launches return
// at once.  The column chunk of the tasks and the number of evaluation workgroups follow the number
// of client pairs, so that few clients still fill the chip.
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
constexpr int kFlagBlock = 256;          // grid_flag_kernel: kFlagGrid workgroups per scenario
#ifndef MMBP_GRID_FLAG_BLOCKS
#define MMBP_GRID_FLAG_BLOCKS 64
#endif
constexpr int kFlagGrid = MMBP_GRID_FLAG_BLOCKS;
static_assert(kFlagGrid <= 64, "one wave of the selection kernel combines the workgroups of grid_flag_kernel");
constexpr int kColChunk = 1024;          // columns staged in LDS per task, at most
constexpr int kMinColChunk = 128;        // the host picks the chunk (a power of two in between) so that few clients still
                                         // give the evaluation enough tasks to fill the chip
constexpr int kRowBlockSegs = (kEvalBlock / kWave) * kRMax;   // 16 segments = 1024 rows per task
constexpr int kMaxPassLaunches = MMBP_GRID_MAX_PASSES;   // the host refuses larger pass limits for this path
constexpr uint32_t kNoJob32 = 0xFFFFFFFFu;
#ifndef MMBP_GRID_FLAG_CAP
#define MMBP_GRID_FLAG_CAP 256
#endif
constexpr int kFlagCap = MMBP_GRID_FLAG_CAP;   // flagged jobs listed in LDS when the first batch of a swap selection fails
static_assert(kSelWaves * 4 == kWave, "one candidate per lane in the selection of a batch");

struct GCtrl {
    unsigned long long evals, pairs_per_scan;
    int egrid;                                 // workgroups of the evaluation kernel (each leaves its candidate count)
    uint32_t vswap, vmove;
    uint32_t bjob[4];                          // first batch of a swap selection (grid_flag_kernel)
    Top3 top;
    int P, nfeas, ntask, passes, status, stop, iters, prune, rk, cchunk;
};

struct GTask {
    uint32_t xy;        // X | Y << 8 | nseg << 16 | rows << 21   (row client, column client, row segments, jobs in the row block)
    uint32_t xrow0;     // first row position
    uint32_t ycol0;     // first column position
    uint32_t yncols;    // columns (multiple of 8) | jobs in the column chunk << 16
};

// what one workgroup of grid_flag_kernel found in its share of the layout
struct FlagPart {
    uint32_t part[4];   // lowest partner of each job of the first batch
    uint32_t k0job;     // lowest flagged job
    uint32_t nflag;     // flagged jobs
    uint32_t spare[2];
};

__host__ __device__ inline size_t up256(size_t x) { return (x + 255) / 256 * 256; }

struct GLayout {        // byte offsets inside one scenario's workspace slice
    size_t ctrl, load, cnt, gstart, feas, cu, job, rowkey, pos, seg_grp, tasks, fpart, ecount, total;
    int pmax, pstride, tmax;
};

__host__ __device__ inline GLayout grid_layout(int N, int M)
{
    GLayout g;
    g.pmax = N + 64 * M;
    g.pstride = (g.pmax + 63) & ~63;
    g.tmax = (g.pmax / 1024 + M) * (N / kMinColChunk + M);
    size_t o = 0;
    g.ctrl = o; o += up256(sizeof(GCtrl));
    g.load = o; o += up256(8 * (size_t)M);
    g.cnt = o; o += up256(4 * (size_t)(M + 1));
    g.gstart = o; o += up256(4 * (size_t)(M + 1));
    g.feas = o; o += up256(4 * (size_t)(M + 1));
    g.cu = o; o += up256(4 * (size_t)g.pmax);
    g.job = o; o += up256(4 * (size_t)g.pmax);
    g.rowkey = o; o += up256(2 * 4 * (size_t)g.pstride);   // two buffers, used by alternate passes
    g.pos = o; o += up256(4 * (size_t)N);
    g.seg_grp = o; o += up256((size_t)g.pmax / 64 + 1);
    g.tasks = o; o += up256(sizeof(GTask) * (size_t)g.tmax);
    g.fpart = o; o += up256(sizeof(FlagPart) * (size_t)kFlagGrid);
    g.ecount = o; o += up256(sizeof(unsigned long long) * (size_t)kEvalGrid);
    g.total = o;
    return g;
}

struct GWs {
    GCtrl *ctrl;
    long long *load;
    int *cnt, *gstart, *feas;
    uint32_t *cu, *job, *pos;            // pos: job -> position in the layout
    uint32_t *rowkey, *rowkey_other;     // per-row minima of this pass; the buffer of the next pass
    uint8_t *seg_grp;
    GTask *tasks;
    FlagPart *fpart;
    unsigned long long *ecount;          // per evaluation workgroup: candidates it evaluated in this scan
    int pmax, pstride, tmax;
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
    w.rowkey = (uint32_t *)(b + g.rowkey) + (size_t)(w.ctrl->rk & 1) * g.pstride;
    w.rowkey_other = (uint32_t *)(b + g.rowkey) + (size_t)((w.ctrl->rk & 1) ^ 1) * g.pstride;
    w.pos = (uint32_t *)(b + g.pos);
    w.seg_grp = (uint8_t *)(b + g.seg_grp);
    w.tasks = (GTask *)(b + g.tasks);
    w.fpart = (FlagPart *)(b + g.fpart);
    w.ecount = (unsigned long long *)(b + g.ecount);
    w.pmax = g.pmax;
    w.tmax = g.tmax;
    w.pstride = g.pstride;
    return w;
}

struct OutPtrs {
    int64_t *load_out, *makespan_out;
    int32_t *passes_out, *status_out;
    uint64_t *evals_out, *applied_log;
};

// Layouts up to this many positions are scanned by the selection workgroup itself (a pass is then
// two launches); larger ones get grid_flag_kernel.
#ifndef MMBP_GRID_SMALL_LAYOUT
#define MMBP_GRID_SMALL_LAYOUT 8192
#endif
inline bool grid_has_flag(int N, int M) { return grid_layout(N, M).pmax > MMBP_GRID_SMALL_LAYOUT; }

// ---- pieces of the one-workgroup kernels (kSelBlock threads, all call) ----

// group the jobs by client: layout starts, segment -> client map, feasible move targets, pair count
// (s_cursor: M ints, s_start: M + 1 ints of LDS; all threads of the workgroup call)
template <typename CostT>
__device__ void g_build_layout(const GWs &w, const CostT *__restrict__ c, const int32_t *asg, int N, int M, int cap,
                               int *s_cursor, int *s_start)
{
    const int tid = threadIdx.x, lane = tid & 63;
    const int pcap = w.pmax & ~63;                        // the blocks are 64 slots wide and end inside the layout
    if (tid < kWave) {
        // wave 0: exclusive prefix of the clients' slot counts, 64 clients per step
        int running = 0, nf = 0;
        unsigned long long sq = 0;
        for (int j0 = 0; j0 < M; j0 += kWave) {
            const int j = j0 + lane;
            const int n = j < M ? min(max(w.cnt[j], 0), N) : 0;
            const int slots = ((n + 63) >> 6) * 64;
            int incl = slots;
            for (int off = 1; off < kWave; off <<= 1) {
                const int up = __shfl_up(incl, off);
                if (lane >= off) incl += up;
            }
            const int start = min(running + incl - slots, pcap);
            if (j < M) { s_start[j] = start; w.gstart[j] = start; }
            running += __builtin_amdgcn_readlane(incl, kWave - 1);
            const bool ok = j < M && n < cap;             // move targets, ascending
            const unsigned long long m = __ballot(ok);
            if (ok) w.feas[nf + __popcll(m & ((1ull << lane) - 1ull))] = j;
            nf += __popcll(m);
            sq += (unsigned long long)n * (unsigned long long)n;
        }
        for (int off = 32; off >= 1; off >>= 1) sq += __shfl_xor(sq, off);
        if (lane == 0) {
            const int P = min(running, pcap);
            s_start[M] = P; w.gstart[M] = P;
            w.ctrl->P = P;
            w.ctrl->nfeas = nf;
            w.ctrl->pairs_per_scan = ((unsigned long long)N * (unsigned long long)N - sq) / 2ull;
        }
    }
    for (int j = tid; j < M; j += kSelBlock) s_cursor[j] = 0;
    __syncthreads();
    const int P = s_start[M];
    for (int sg = tid; sg < (P >> 6); sg += kSelBlock) {  // segment -> client: the last client starting at or before it
        const int pos = sg << 6;                          // (clients without jobs share a start with their successor)
        int lo = 0, hi = M;                               // first client whose start exceeds pos
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (s_start[mid] <= pos) lo = mid + 1; else hi = mid;
        }
        w.seg_grp[sg] = (uint8_t)max(lo - 1, 0);
    }
    {
        uint4 *cu4 = (uint4 *)w.cu, *jb4 = (uint4 *)w.job;
        for (int q = tid; q < (P >> 2); q += kSelBlock) {
            cu4[q] = make_uint4(kPad, kPad, kPad, kPad);
            jb4[q] = make_uint4(kNoJob32, kNoJob32, kNoJob32, kNoJob32);
        }
    }
    __syncthreads();
    for (int i = tid; i < N; i += kSelBlock) {
        const int a = asg[i];
        const int p = s_start[a] + atomicAdd(&s_cursor[a], 1);
        if (p < P) { w.cu[p] = 2u * (uint32_t)c[i] + kBias; w.job[p] = (uint32_t)i; }
        w.pos[i] = (uint32_t)min(p, P - 1);
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
__device__ bool g_prep_pass(const GWs &w, const OutPtrs &o, int s, int M, int max_passes, bool last_launch,
                            bool toggle, int *s_ntask)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    GCtrl *ctrl = w.ctrl;
    if (wave == 0) {
        // (the control fields are fetched before the top-3 reduction and used after it, so that
        // their latency overlaps with the loads of the reduction)
        int iters = 0, stop = 0, passes = 0, rk = 0;
        if (lane == 0) { iters = ctrl->iters + 1; stop = ctrl->stop; passes = ctrl->passes; rk = ctrl->rk; }
        const Top3 t = wave_top3(w.load, M, lane);
        if (lane == 0) {
            ctrl->iters = iters;
            if ((long long)iters > (long long)max_passes + 1) { ctrl->status = MMBP_ST_INTERNAL; ctrl->stop = 1; }
            else if (stop) { }
            else if (passes == max_passes || last_launch) { ctrl->status = MMBP_ST_TRUNCATED; ctrl->stop = 1; }
            ctrl->vswap = kInf; ctrl->vmove = kInf;
            if (toggle) ctrl->rk = (rk & 1) ^ 1;         // the other buffer has been reset for the next pass
            *s_ntask = 0;
            ctrl->top = t;
        }
    }
    __syncthreads();
    if (ctrl->stop) { g_finish(w, o, s, M); return false; }
    __shared__ int s_cn[MMBP_MAX_M], s_gs[MMBP_MAX_M];
    __shared__ int s_single;                             // every client is non-empty, one row block and one column chunk
    const int prune = ctrl->prune;
    const int cchunk = min(max(ctrl->cchunk, kMinColChunk), kColChunk) & ~7;
    if (tid == 0) s_single = 1;
    __syncthreads();
    for (int j = tid; j < M; j += kSelBlock) {
        const int n = w.cnt[j];
        s_cn[j] = n; s_gs[j] = w.gstart[j];
        if (n <= 0 || n > kRowBlockSegs * 64 || ((n + 7) & ~7) > cchunk) s_single = 0;
    }
    __syncthreads();
    // task table: every unordered pair of non-empty clients once, the critical client as columns
    const int astar = min(max(ctrl->top.j0, 0), M - 1);
    // Two rounds: the first task of every pair (a full row block x a full column chunk unless the
    // pair is smaller), then the remainders, so that the stride loop of the evaluation gives every
    // workgroup the same number of large tasks.
    if (s_single && !prune) {
        // Every pair of clients is exactly one task: its slot follows from the pair (the pairs (g, b),
        // g < b, in row-major order), so the table needs no slot reservation and no second round.
        for (int q = tid; q < M * M; q += kSelBlock) {
            const int g = q / M, b = q - g * M;
            if (g >= b) continue;
            const int X = (g == astar) ? b : g, Y = (g == astar) ? g : b;
            const int nx = s_cn[X], ny = s_cn[Y];
            GTask e;
            e.xy = (uint32_t)X | ((uint32_t)Y << 8) | ((uint32_t)((nx + 63) >> 6) << 16) | ((uint32_t)nx << 21);
            e.xrow0 = (uint32_t)s_gs[X];
            e.ycol0 = (uint32_t)s_gs[Y];
            e.yncols = (uint32_t)((ny + 7) & ~7) | ((uint32_t)ny << 16);
            const int slot = g * M - (g * (g + 1)) / 2 + (b - g - 1);
            if (slot < w.tmax) w.tasks[slot] = e;        // (always: tmax bounds the table)
        }
        if (tid == 0) ctrl->ntask = min(M * (M - 1) / 2, w.tmax);
        return true;
    }
    __shared__ int s_more;                               // some pair has more than one task
    if (tid == 0) s_more = 0;
    __syncthreads();
    for (int round = 0; round < 2; round++) {
        if (round == 1 && !s_more) break;                // the usual case with balanced clients: one task per pair
        for (int q0 = 0; q0 < M * M; q0 += kSelBlock) {  // uniform trip count: the waves cooperate below
            const int q = q0 + tid;
            const int g = q / M, b = q - g * M;
            const bool pair = q < M * M && g < b && !(prune && g != astar && b != astar);   // pruned scan: pairs
            const int X = (g == astar) ? b : g, Y = (g == astar) ? g : b;                      // with the critical client only
            const int nx = pair ? s_cn[X] : 0, ny = pair ? s_cn[Y] : 0;
            const int segx = (nx + 63) >> 6;
            const int nrb = (segx + kRowBlockSegs - 1) / kRowBlockSegs;
            const int ncols = (ny + 7) & ~7;
            const int ncc = (ncols + cchunk - 1) / cchunk;
            const int all = (nx > 0 && ny > 0) ? nrb * ncc : 0;
            const int mine = round == 0 ? min(all, 1) : max(all - 1, 0);
            if (round == 0 && all > 1) s_more = 1;
            int incl = mine;                              // one slot reservation per wave
            for (int off = 1; off < kWave; off <<= 1) {
                const int up = __shfl_up(incl, off);
                if (lane >= off) incl += up;
            }
            const int total = __builtin_amdgcn_readlane(incl, kWave - 1);
            int wbase = 0;
            if (lane == 0 && total > 0) wbase = atomicAdd(s_ntask, total);
            wbase = __builtin_amdgcn_readfirstlane(wbase);
            int slot = wbase + incl - mine;
            if (mine == 0 || slot + mine > w.tmax) continue;   // (the second cannot happen: tmax bounds the table)
            for (int rb = 0; rb < nrb; rb++)
                for (int cc = 0; cc < ncc; cc++) {
                    if ((rb == 0 && cc == 0) != (round == 0)) continue;
                    GTask e;
                    e.xy = (uint32_t)X | ((uint32_t)Y << 8) | ((uint32_t)min(kRowBlockSegs, segx - rb * kRowBlockSegs) << 16) |
                           ((uint32_t)min(kRowBlockSegs * 64, nx - rb * kRowBlockSegs * 64) << 21);
                    e.xrow0 = (uint32_t)(s_gs[X] + rb * kRowBlockSegs * 64);
                    e.ycol0 = (uint32_t)(s_gs[Y] + cc * cchunk);
                    e.yncols = (uint32_t)min(cchunk, ncols - cc * cchunk) | ((uint32_t)min(cchunk, ny - cc * cchunk) << 16);
                    w.tasks[slot++] = e;
                }
        }
        __syncthreads();                                  // all first tasks are placed before any remainder
    }
    __syncthreads();
    if (tid == 0) ctrl->ntask = min(*s_ntask, w.tmax);
    return true;
}

// ---- kernel 0: validation, narrowing decision, layout, first pass preparation ----
template <typename CostT>
__global__ __launch_bounds__(kSelBlock) void grid_stage_kernel(const CostT *__restrict__ cost_all, int N, int M, int cap,
                                                               int max_passes, int prune, int cchunk, int egrid,
                                                               int32_t *assign_all, OutPtrs o, void *workspace)
{
    const int s = blockIdx.x;
    const GWs w = grid_ws(workspace, s, N, M);
    GCtrl *ctrl = w.ctrl;
    const CostT *c = cost_all + (size_t)s * N;
    const int32_t *asg = assign_all + (size_t)s * N;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    __shared__ long long s_load[MMBP_MAX_M];
    __shared__ int s_cnt[MMBP_MAX_M], s_start[MMBP_MAX_M + 1];
    __shared__ unsigned long long s_wsum[kSelWaves], s_wmax[kSelWaves];
    __shared__ int s_bad_cost, s_bad_assign, s_ntask;
    __shared__ long long s_T0;

    for (int j = tid; j < M; j += kSelBlock) { s_load[j] = 0; s_cnt[j] = 0; }
    if (tid == 0) {
        s_bad_cost = 0; s_bad_assign = 0;
        ctrl->passes = 0; ctrl->status = MMBP_ST_OK; ctrl->stop = 0; ctrl->evals = 0; ctrl->iters = 0; ctrl->ntask = 0;
        ctrl->prune = prune; ctrl->rk = 0; ctrl->cchunk = cchunk; ctrl->egrid = egrid;
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
    g_build_layout<CostT>(w, c, asg, N, M, cap, s_cnt /* reused as cursors */, s_start);
    {
        uint4 *rk4 = (uint4 *)(w.rowkey < w.rowkey_other ? w.rowkey : w.rowkey_other);   // both buffers
        for (int q = tid; q < (w.pstride >> 1); q += kSelBlock) rk4[q] = make_uint4(kInf, kInf, kInf, kInf);
    }
    g_prep_pass(w, o, s, M, max_passes, false, false, &s_ntask);
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

__global__ __launch_bounds__(kEvalBlock, 8) void grid_eval_kernel(int N, int M, void *workspace)
{
    const int s = blockIdx.y;
    const GWs w = grid_ws(workspace, s, N, M);
    GCtrl *ctrl = w.ctrl;
    if (ctrl->stop) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    __shared__ __align__(16) uint32_t cols[kColChunk];
    __shared__ uint32_t s_ld[MMBP_MAX_M];
    __shared__ int s_feas[MMBP_MAX_M];
    Top3 top;
    top.v0 = uniu(ctrl->top.v0); top.v1 = uniu(ctrl->top.v1); top.v2 = uniu(ctrl->top.v2);
    top.j0 = uni(ctrl->top.j0); top.j1 = uni(ctrl->top.j1); top.j2 = uni(ctrl->top.j2);
    const int astar = min(max(top.j0, 0), M - 1);
    const int ntask = min(ctrl->ntask, w.tmax);
    const int P = min(ctrl->P, w.pmax);
    const int nfeas = min(ctrl->nfeas, M);
    uint32_t sbest = kInf, mbest = kInf;
    unsigned long long ecnt = 0, mcnt = 0;      // candidates of this workgroup's tasks (uniform) and of this wave's move segments
    for (int j = tid; j < M; j += kEvalBlock) { s_ld[j] = (uint32_t)w.load[j]; s_feas[j] = j < nfeas ? w.feas[j] : 0; }
    __syncthreads();

    // (a shared counter dealing the tasks out on demand was measured slower: thousands of atomics
    // on one address take longer than the imbalance they remove; the table lists the full-size
    // tasks first instead, so the stride gives every workgroup the same number of them)
    for (int t = blockIdx.x; t < ntask; t += gridDim.x) {
        const GTask e = w.tasks[t];
        const int X = (int)(e.xy & 0xFFu), Y = (int)((e.xy >> 8) & 0xFFu), nseg = min((int)((e.xy >> 16) & 0x1Fu), kRowBlockSegs);
        const int ncols = min((int)(e.yncols & 0xFFFFu), kColChunk) & ~7;
        ecnt += (unsigned long long)(e.xy >> 21) * (unsigned long long)(e.yncols >> 16);     // jobs in the row block x jobs in the chunk
        const int ycol0 = max(min((int)e.ycol0, w.pmax - ncols), 0);
        for (int i = tid; i < ncols; i += kEvalBlock) cols[i] = w.cu[ycol0 + i];
        __syncthreads();
        const int role = (wave + t) & (kEvalBlock / kWave - 1);   // short row blocks: not always the same SIMD
        const int rowbase = (int)e.xrow0 + role * kRMax * 64;
        int R = min(max(nseg - role * kRMax, 0), kRMax);
        if (rowbase < 0 || rowbase + 64 * R > w.pmax) R = 0;      // cannot happen: rows lie inside the layout
        if (R > 0 && ncols > 0) {
            const uint32_t lx = s_ld[X], ly = s_ld[Y];
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
    if (nfeas > 0) {
        const int nseg = P >> 6;
        for (int seg = blockIdx.x * (kEvalBlock / kWave) + wave; seg < nseg; seg += gridDim.x * (kEvalBlock / kWave)) {
            const int g = w.seg_grp[seg];
            if (ctrl->prune && g != astar) continue;                 // an improving move leaves the critical client
            const uint32_t x = w.cu[seg * 64 + lane];
            const uint32_t ci = (x - kBias) >> 1;
            const uint32_t la = s_ld[g];
            mcnt += (unsigned long long)__popcll(__ballot(x != kPad)) * (unsigned long long)(M - 1);
            uint32_t m = kInf;
            for (int q = 0; q < nfeas; q++) {
                const int b = s_feas[q];
                if (b == g) continue;
                m = min(m, max(max(la - ci, s_ld[b] + ci), others_max(top, g, b)));
            }
            if (x != kPad) mbest = min(mbest, m);
        }
    }
    // One atomic per workgroup and kind at most, and none when the control block already holds a
    // value as low (the plain read may be stale, i.e. too high: then the atomic is merely redundant).
    // Atomics of thousands of waves on one address would cost more than the evaluation's tail.
    mbest = wave_min_u32(mbest);
    sbest = wave_min_u32(sbest);
    __shared__ uint32_t s_wm[kEvalBlock / kWave], s_ws[kEvalBlock / kWave];
    __shared__ unsigned long long s_wc[kEvalBlock / kWave];
    if (lane == 0) { s_wm[wave] = mbest; s_ws[wave] = sbest; s_wc[wave] = mcnt; }
    __syncthreads();
    if (tid == 0) {
        for (int q = 0; q < kEvalBlock / kWave; q++) ecnt += s_wc[q];
        w.ecount[blockIdx.x] = ecnt;                     // plain store, every workgroup: the selection kernel adds them up
        for (int q = 1; q < kEvalBlock / kWave; q++) { mbest = min(mbest, s_wm[q]); sbest = min(sbest, s_ws[q]); }
        if (mbest < __hip_atomic_load(&ctrl->vmove, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMin(&ctrl->vmove, mbest);
        if (sbest < __hip_atomic_load(&ctrl->vswap, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMin(&ctrl->vswap, sbest);
    }
}

// ---- exact selection of a swap: pieces shared by grid_flag_kernel and grid_select_kernel ----
// Every swap of the best value V pairs a job of the critical client with a flagged job (row
// minimum == V) of another client.  With k0 the flagged job of lowest index, the lowest
// (min(i,k), max(i,k)) is either (e, f) for the lowest critical job e < k0 that has a partner (f its
// lowest partner), or (k0, c) with c the lowest critical partner of k0.  Ties at V are the rule on
// large instances (V is often the load of the second client), so the flagged jobs are not listed:
// one pass over the layout finds k0 and, for the four critical jobs of lowest index, their lowest
// partners (grid_flag_kernel, many workgroups).  When that does not settle it, a short list of
// flagged jobs is tried against all early critical jobs; with a long list, batches of four go on.
struct SwapCtx {
    const uint32_t *ld;        // loads of the clients (LDS copy)
    Top3 top;
    uint32_t V, lstar;
    int astar, sbase, send, sslots, P;   // critical client: its jobs [sbase, send), its slots up to sslots
};

__device__ __forceinline__ SwapCtx swap_ctx(const GWs &w, const uint32_t *ld, const Top3 &top, uint32_t V, int astar, int P)
{
    SwapCtx c;
    c.ld = ld; c.top = top; c.V = V; c.astar = astar; c.P = P;
    c.lstar = ld[astar];
    c.sbase = min(max(w.gstart[astar], 0), P);
    const int scnt = min(max(w.cnt[astar], 0), P - c.sbase);
    c.send = c.sbase + scnt;
    c.sslots = c.sbase + ((scnt + 63) & ~63);
    return c;
}

// A pair (critical job e, job f of client g) reaches V exactly when its key |cu_e - (cu_f - sh)|
// lies in [klo, klo + span], i.e. max(others, (l_g + l_star + key) >> 1) == V.  False: no key does
// (the range returned then is meaningless).
__device__ __forceinline__ bool key_range(const SwapCtx &c, int g, uint32_t &sh, uint32_t &klo, uint32_t &span)
{
    const uint32_t lg = c.ld[g], lsum = lg + c.lstar, oth = others_max(c.top, g, c.astar);
    sh = lg - c.lstar;
    // (lsum + key) >> 1 <= V  <=>  key <= 2V + 1 - lsum; compared in 64 bits: the difference can be
    // negative (a client too loaded for any swap with the critical one to reach V)
    const long long room = 2ll * (long long)c.V + 1ll - (long long)lsum;
    const bool reach = oth <= c.V && room >= 0;
    const uint32_t khi = (uint32_t)min(max(room, 0ll), (long long)(kKeyLimit - 1u));
    klo = (oth == c.V || room < 1) ? 0u : (uint32_t)(room - 1);     // below V the value must be exactly V
    const bool some = reach && klo <= khi;
    klo = some ? klo : 0u;                                          // none: the caller masks on the result
    span = some ? khi - klo : 0u;
    return some;
}

// The four critical jobs of lowest index (above `last` when `after`), ascending, kNoJob32 for
// none.  All threads of the workgroup call; s_cand holds 4 entries per wave (at most 16 waves);
// contains one barrier, and the caller separates two calls by another.
__device__ void lowest_four(const GWs &w, const SwapCtx &c, bool after, uint32_t last, uint32_t *s_cand, uint32_t bjob[4])
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nwave = (int)(blockDim.x >> 6);
    uint32_t m0 = kNoJob32, m1 = kNoJob32, m2 = kNoJob32, m3 = kNoJob32;
    for (int p = c.sbase + tid; p < c.send; p += (int)blockDim.x) {
        const uint32_t jb = w.job[p];
        if ((after && jb <= last) || jb >= m3) continue;
        m3 = jb;
        if (m3 < m2) { const uint32_t t = m2; m2 = m3; m3 = t; }
        if (m2 < m1) { const uint32_t t = m1; m1 = m2; m2 = t; }
        if (m1 < m0) { const uint32_t t = m0; m0 = m1; m1 = t; }
    }
    uint32_t mine = kNoJob32;
#pragma unroll
    for (int r = 0; r < 4; r++) {
        const uint32_t mw = wave_min_u32(m0);
        if (lane == r) mine = mw;
        if (m0 == mw && m0 != kNoJob32) { m0 = m1; m1 = m2; m2 = m3; m3 = kNoJob32; }
    }
    if (lane < 4) s_cand[wave * 4 + lane] = mine;
    __syncthreads();
    uint32_t v = lane < nwave * 4 ? s_cand[lane] : kNoJob32;
#pragma unroll
    for (int r = 0; r < 4; r++) {
        bjob[r] = wave_min_u32(v);
        if (v == bjob[r]) v = kNoJob32;
    }
}

// Layout positions outside the critical client, four per step from quad q0 with stride qstride:
// per batch job r the lowest partner pm[r]; from the row minima (rowkey != nullptr) the lowest
// flagged job k0 and the number of flagged jobs.  Results are per lane (the caller reduces).
__device__ __forceinline__ void scan_partners(const GWs &w, const SwapCtx &c, const uint32_t *rowkey, const uint32_t bx[4],
                                              int q0, int qstride, uint32_t pm[4], uint32_t &k0, uint32_t &nflag)
{
    const uint4 *rk4 = (const uint4 *)rowkey, *cu4 = (const uint4 *)w.cu, *jb4 = (const uint4 *)w.job;
    const int nquad = c.P >> 2;
    for (int q = q0; q < nquad; q += qstride) {
        const int p = q << 2;
        if (p >= c.sbase && p < c.sslots) continue;
        uint4 r4 = make_uint4(kInf, kInf, kInf, kInf);
        if (rowkey) r4 = rk4[q];
        uint32_t sh, klo, span;
        const bool reach = key_range(c, w.seg_grp[p >> 6], sh, klo, span);
        if (!reach && !rowkey) continue;                  // no job of this client reaches V
        const uint4 x4 = cu4[q], j4 = jb4[q];
        const uint32_t xs[4] = {x4.x, x4.y, x4.z, x4.w}, js[4] = {j4.x, j4.y, j4.z, j4.w};
        const uint32_t rs[4] = {r4.x, r4.y, r4.z, r4.w};
#pragma unroll
        for (int e = 0; e < 4; e++) {                      // padding slots carry kNoJob32: harmless in a min
            const uint32_t xf = xs[e] - sh, j = reach ? js[e] : kNoJob32;
            if (rs[e] == c.V) { k0 = min(k0, js[e]); nflag += 1; }
#pragma unroll
            for (int r = 0; r < 4; r++) pm[r] = min(pm[r], __usad(bx[r], xf, 0u) - klo <= span ? j : kNoJob32);
        }
    }
}

// ---- kernel 2: first step of the selection of a swap, and reset of the next pass's row minima ----
__global__ __launch_bounds__(kFlagBlock) void grid_flag_kernel(int N, int M, void *workspace)
{
    const int s = blockIdx.y;
    const GWs w = grid_ws(workspace, s, N, M);
    GCtrl *ctrl = w.ctrl;
    if (ctrl->stop) return;
    const int tid = threadIdx.x, lane = tid & 63;
    const int gtid = (int)blockIdx.x * kFlagBlock + tid, gthreads = (int)gridDim.x * kFlagBlock;
    {
        uint4 *o4 = (uint4 *)w.rowkey_other;
        for (int q = gtid; q < (w.pstride >> 2); q += gthreads) o4[q] = make_uint4(kInf, kInf, kInf, kInf);
    }
    Top3 top;
    top.v0 = uniu(ctrl->top.v0); top.v1 = uniu(ctrl->top.v1); top.v2 = uniu(ctrl->top.v2);
    top.j0 = uni(ctrl->top.j0); top.j1 = uni(ctrl->top.j1); top.j2 = uni(ctrl->top.j2);
    const uint32_t Vm = ctrl->vmove, Vs = ctrl->vswap;
    if (Vs >= top.v0 || Vm <= Vs) return;                // local optimum, or a move wins
    __shared__ uint32_t s_ld[MMBP_MAX_M], s_cand[(kFlagBlock / kWave) * 4];
    for (int j = tid; j < M; j += kFlagBlock) s_ld[j] = (uint32_t)w.load[j];
    __syncthreads();
    const int astar = min(max(top.j0, 0), M - 1);
    const SwapCtx c = swap_ctx(w, s_ld, top, Vs, astar, min(ctrl->P, w.pmax));
    uint32_t bjob[4], bx[4];
    lowest_four(w, c, false, 0u, s_cand, bjob);
#pragma unroll
    for (int r = 0; r < 4; r++) bx[r] = bjob[r] < (uint32_t)N ? w.cu[min((int)w.pos[bjob[r]], c.P - 1)] : kPad;
    uint32_t pm[4] = {kNoJob32, kNoJob32, kNoJob32, kNoJob32}, k0 = kNoJob32, nflag = 0;
    scan_partners(w, c, w.rowkey, bx, gtid, gthreads, pm, k0, nflag);
#pragma unroll
    for (int r = 0; r < 4; r++) pm[r] = wave_min_u32(pm[r]);
    k0 = wave_min_u32(k0);
    for (int off = 32; off >= 1; off >>= 1) nflag += __shfl_xor(nflag, off);
    __shared__ uint32_t s_red[kFlagBlock / kWave][6];
    if (lane == 0) {
        uint32_t *row = s_red[tid >> 6];
        row[0] = pm[0]; row[1] = pm[1]; row[2] = pm[2]; row[3] = pm[3]; row[4] = k0; row[5] = nflag;
    }
    __syncthreads();
    if (tid < 6) {                                       // plain stores: the selection kernel combines the workgroups
        uint32_t v = s_red[0][tid];
        for (int q = 1; q < kFlagBlock / kWave; q++) v = tid < 5 ? min(v, s_red[q][tid]) : v + s_red[q][tid];
        uint32_t *out = (uint32_t *)&w.fpart[blockIdx.x];
        out[tid] = v;
    }
    if (blockIdx.x == 0 && tid < 4) ctrl->bjob[tid] = tid == 0 ? bjob[0] : tid == 1 ? bjob[1] : tid == 2 ? bjob[2] : bjob[3];
}

// ---- kernel 3: exact selection, apply, preparation of the next pass ----
template <typename CostT>
__global__ __launch_bounds__(kSelBlock) void grid_select_kernel(const CostT *__restrict__ cost_all, int N, int M, int cap,
                                                                int max_passes, int32_t *assign_all, OutPtrs o,
                                                                void *workspace, int last_launch, int has_flag)
{
    const int s = blockIdx.x;
    const GWs w = grid_ws(workspace, s, N, M);
    GCtrl *ctrl = w.ctrl;
    if (ctrl->stop) return;
    if (!has_flag) {                                     // no grid_flag_kernel in this mode: its other duty
        uint4 *o4 = (uint4 *)w.rowkey_other;
        for (int q = threadIdx.x; q < (w.pstride >> 2); q += kSelBlock) o4[q] = make_uint4(kInf, kInf, kInf, kInf);
    }
    const CostT *c = cost_all + (size_t)s * N;
    int32_t *asg = assign_all + (size_t)s * N;
    const int tid = threadIdx.x, lane = tid & 63;
    __shared__ int s_cursor[MMBP_MAX_M], s_start[MMBP_MAX_M + 1];
    __shared__ uint32_t s_ld[MMBP_MAX_M];
    __shared__ int s_feas[MMBP_MAX_M];
    __shared__ int s_ntask, s_rebuild;
    __shared__ unsigned long long s_best;
    __shared__ uint32_t s_later, s_part[4], s_cand[kSelWaves * 4];
    __shared__ int s_nlist;
    __shared__ FlagPart s_flag;
    __shared__ uint32_t s_fpos[kFlagCap], s_fx[kFlagCap], s_fklo[kFlagCap], s_fspan[kFlagCap], s_fjob[kFlagCap];

    Top3 top;
    top.v0 = uniu(ctrl->top.v0); top.v1 = uniu(ctrl->top.v1); top.v2 = uniu(ctrl->top.v2);
    top.j0 = uni(ctrl->top.j0); top.j1 = uni(ctrl->top.j1); top.j2 = uni(ctrl->top.j2);
    const uint32_t T = top.v0;
    const int astar = min(max(top.j0, 0), M - 1);
    const int P = min(ctrl->P, w.pmax);
    const int nfeas = min(ctrl->nfeas, M);
    const uint32_t Vm = ctrl->vmove, Vs = ctrl->vswap;
    const uint32_t V = min(Vm, Vs);
    if (tid == 0) { s_rebuild = 0; s_later = kNoJob32; s_nlist = 0; s_best = ~0ull; }
    for (int j = tid; j < M; j += kSelBlock) { s_ld[j] = (uint32_t)w.load[j]; s_feas[j] = j < nfeas ? w.feas[j] : 0; }
    // The candidates of the scan just run: N (M - 1) moves and every pair on different clients.  The
    // full scan adds up what its evaluation workgroups counted (moves whose targets are all full are the
    // uniform capacity test: counted here) and stops the scenario if that is not the whole
    // neighbourhood; the pruned scan reports that number by definition.
    __shared__ unsigned long long s_cnt[kSelWaves];
    bool count_short;
    {
        // (the control words are fetched before the reduction so that their latency overlaps with it)
        const unsigned long long pairs = ctrl->pairs_per_scan;
        const int prune = ctrl->prune;
        const unsigned long long ev0 = tid == 0 ? ctrl->evals : 0ull;
        unsigned long long part = 0;
        const int eg = min(max(ctrl->egrid, 0), kEvalGrid);
        if (!prune)
            for (int q = tid; q < eg; q += kSelBlock) part += w.ecount[q];
        for (int off = 32; off >= 1; off >>= 1) part += __shfl_xor(part, off);
        if (lane == 0) s_cnt[tid >> 6] = part;
        __syncthreads();
        const unsigned long long moves = (unsigned long long)N * (unsigned long long)(M - 1);
        const unsigned long long whole = moves + pairs;
        unsigned long long counted = nfeas == 0 ? moves : 0ull;
#pragma unroll
        for (int q = 0; q < kSelWaves; q++) counted += s_cnt[q];
        if (prune) counted = whole;
        count_short = counted != whole;                  // the same in every thread: all read the same words
        if (tid == 0) {
            ctrl->evals = ev0 + counted;
            if (count_short) ctrl->status = MMBP_ST_INTERNAL;
        }
    }
    if (count_short) {                                   // cannot happen: the task table covers every client pair
        g_finish(w, o, s, M);
        return;
    }
    if (V >= T) {                                        // local optimum
        g_finish(w, o, s, M);
        return;
    }
    if (Vm <= Vs) {
        // A move wins: the lowest id among the moves of value V.  V is below the makespan, so the
        // job leaves the critical client: only its jobs are scanned.
        const int sbase = min(max(w.gstart[astar], 0), P), send = sbase + min(max(w.cnt[astar], 0), P - sbase);
        const uint32_t la = s_ld[astar];
        unsigned long long best = ~0ull;
        for (int p = sbase + tid; p < send; p += kSelBlock) {
            const uint32_t x = w.cu[p], jb = w.job[p];
            if (x == kPad) continue;
            const uint32_t ci = (x - kBias) >> 1;
            for (int q = 0; q < nfeas; q++) {
                const int b = s_feas[q];
                if (b == astar) continue;
                const uint32_t v = max(max(la - ci, s_ld[b] + ci), others_max(top, astar, b));
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
            if (mv == ~0ull || i >= N || p < sbase || p >= send) { ctrl->status = MMBP_ST_INTERNAL; ctrl->stop = 1; }
            else {
                const int a = astar, na = w.cnt[a], nb = w.cnt[b];
                const uint32_t x = w.cu[p];
                const long long ci = (long long)((x - kBias) >> 1);
                w.load[a] -= ci; w.load[b] += ci;
                w.cnt[a] = na - 1; w.cnt[b] = nb + 1;
                asg[i] = b;
                if (o.applied_log) o.applied_log[(size_t)s * max_passes + ctrl->passes] = (uint64_t)id;
                ctrl->passes += 1;
                // Layout: the last job of the source client fills the hole; the job goes to the first
                // free slot of the target client.  Only a target whose slots are all taken needs the
                // layout rebuilt.  (The order of the jobs inside a client decides nothing.)
                const int slot = w.gstart[b] + nb;
                if (slot >= w.gstart[b + 1]) s_rebuild = 1;
                else {
                    const int last = sbase + na - 1;
                    if (p != last) {
                        const uint32_t jl = w.job[last];
                        w.cu[p] = w.cu[last]; w.job[p] = jl;
                        if (jl < (uint32_t)N) w.pos[jl] = (uint32_t)p;
                    }
                    w.cu[last] = kPad; w.job[last] = kNoJob32;
                    w.cu[slot] = x; w.job[slot] = (uint32_t)i; w.pos[i] = (uint32_t)slot;
                    // unordered pairs on different clients: N^2 - sum n^2 over 2
                    ctrl->pairs_per_scan -= (unsigned long long)((long long)nb - (long long)na + 1);
                }
            }
        }
        __syncthreads();
        if (s_rebuild) g_build_layout<CostT>(w, c, asg, N, M, cap, s_cursor, s_start);
        else if (tid < kWave) {                          // move targets: clients below the cap, ascending
            int nf = 0;
            for (int j0 = 0; j0 < M; j0 += kWave) {
                const int j = j0 + lane;
                const bool ok = j < M && w.cnt[j] < cap;
                const unsigned long long m = __ballot(ok);
                if (ok) w.feas[nf + __popcll(m & ((1ull << lane) - 1ull))] = j;
                nf += __popcll(m);
            }
            if (lane == 0) ctrl->nfeas = nf;
        }
    } else {
        // a swap wins (see above); the first batch was taken by grid_flag_kernel, or is taken here
        const SwapCtx sc = swap_ctx(w, s_ld, top, V, astar, P);
        uint32_t bjob[4], part[4], ji = kNoJob32, jk = kNoJob32;
        if (!has_flag) {                                 // small layout: one workgroup scans it as fast as a launch takes
            if (tid == 0) { s_flag.part[0] = s_flag.part[1] = s_flag.part[2] = s_flag.part[3] = s_flag.k0job = kNoJob32; s_flag.nflag = 0; }
            lowest_four(w, sc, false, 0u, s_cand, bjob);  // (its barrier also publishes the reset of s_flag)
            uint32_t bx[4];
#pragma unroll
            for (int r = 0; r < 4; r++) bx[r] = bjob[r] < (uint32_t)N ? w.cu[min((int)w.pos[bjob[r]], P - 1)] : kPad;
            uint32_t pm[4] = {kNoJob32, kNoJob32, kNoJob32, kNoJob32}, k0 = kNoJob32, nf = 0;
            scan_partners(w, sc, w.rowkey, bx, tid, kSelBlock, pm, k0, nf);
#pragma unroll
            for (int r = 0; r < 4; r++) {
                pm[r] = wave_min_u32(pm[r]);
                if (lane == 0 && pm[r] != kNoJob32) atomicMin(&s_flag.part[r], pm[r]);
            }
            k0 = wave_min_u32(k0);
            for (int off = 32; off >= 1; off >>= 1) nf += __shfl_xor(nf, off);
            if (lane == 0 && k0 != kNoJob32) atomicMin(&s_flag.k0job, k0);
            if (lane == 0 && nf) atomicAdd(&s_flag.nflag, nf);
        } else if (tid < kWave) {                        // combine what the workgroups of grid_flag_kernel found
            FlagPart f;
            f.part[0] = f.part[1] = f.part[2] = f.part[3] = f.k0job = kNoJob32; f.nflag = 0;
            if (lane < kFlagGrid) f = w.fpart[lane];
#pragma unroll
            for (int r = 0; r < 4; r++) f.part[r] = wave_min_u32(f.part[r]);
            f.k0job = wave_min_u32(f.k0job);
            for (int off = 32; off >= 1; off >>= 1) f.nflag += __shfl_xor(f.nflag, off);
            if (lane == 0) s_flag = f;
        }
        __syncthreads();
        const uint32_t k0job = s_flag.k0job, nflag = s_flag.nflag;
        if (k0job >= (uint32_t)N) {                      // cannot happen: a best swap has a flagged job
            if (tid == 0) ctrl->status = MMBP_ST_INTERNAL;
            __syncthreads();
            g_finish(w, o, s, M);
            return;
        }
#pragma unroll
        for (int r = 0; r < 4; r++) { if (has_flag) bjob[r] = ctrl->bjob[r]; part[r] = s_flag.part[r]; }
        bool found = false, early_done = false;
        auto decide = [&]() {
#pragma unroll
            for (int r = 0; r < 4; r++) {
                if (found || early_done) continue;
                if (bjob[r] >= (uint32_t)N || bjob[r] > k0job) { early_done = true; continue; }
                if (part[r] < (uint32_t)N) { found = true; ji = bjob[r]; jk = part[r]; }
            }
        };
        decide();
        while (!found && !early_done && nflag > (uint32_t)kFlagCap) {
            // many flagged jobs and no partner yet: the next four early critical jobs
            const uint32_t last = bjob[3];
            if (tid < 4) s_part[tid] = kNoJob32;
            lowest_four(w, sc, true, last, s_cand, bjob);
            uint32_t bx[4];
#pragma unroll
            for (int r = 0; r < 4; r++) bx[r] = bjob[r] < (uint32_t)N ? w.cu[min((int)w.pos[bjob[r]], P - 1)] : kPad;
            uint32_t pm[4] = {kNoJob32, kNoJob32, kNoJob32, kNoJob32}, k0 = kNoJob32, nf = 0;
            scan_partners(w, sc, nullptr, bx, tid, kSelBlock, pm, k0, nf);
#pragma unroll
            for (int r = 0; r < 4; r++) {
                pm[r] = wave_min_u32(pm[r]);
                if (lane == 0 && pm[r] != kNoJob32) atomicMin(&s_part[r], pm[r]);
            }
            __syncthreads();
#pragma unroll
            for (int r = 0; r < 4; r++) part[r] = s_part[r];
            decide();
            __syncthreads();                             // s_cand, s_part are rewritten by the next batch
        }
        if (!found && !early_done) {
            // few flagged jobs: list them and try all of them against every early critical job
            const uint4 *rk4 = (const uint4 *)w.rowkey;
            for (int q = tid; q < (P >> 2); q += kSelBlock) {
                const int p = q << 2;
                if (p >= sc.sbase && p < sc.sslots) continue;
                const uint4 r4 = rk4[q];
                const uint32_t rs[4] = {r4.x, r4.y, r4.z, r4.w};
#pragma unroll
                for (int e = 0; e < 4; e++)
                    if (rs[e] == V) {
                        const int idx = atomicAdd(&s_nlist, 1);
                        if (idx < kFlagCap) s_fpos[idx] = (uint32_t)(p + e);
                    }
            }
            __syncthreads();
            const int nl = min(s_nlist, kFlagCap);
            if (tid < nl) {
                const int p = min((int)s_fpos[tid], P - 1);
                uint32_t sh, klo, span;
                const bool ok = key_range(sc, w.seg_grp[p >> 6], sh, klo, span);
                s_fx[tid] = w.cu[p] - sh;
                s_fklo[tid] = klo;
                s_fspan[tid] = span;                     // not ok: masked by the job below
                s_fjob[tid] = ok ? w.job[p] : kNoJob32;
            }
            __syncthreads();
            unsigned long long best = ~0ull;
            for (int p = sc.sbase + tid; p < sc.send; p += kSelBlock) {
                const uint32_t jb = w.job[p];
                if (jb >= k0job) continue;
                const uint32_t x = w.cu[p];
                uint32_t pm = kNoJob32;
                for (int f = 0; f < nl; f++)
                    pm = min(pm, __usad(x, s_fx[f], 0u) - s_fklo[f] <= s_fspan[f] ? s_fjob[f] : kNoJob32);
                if (pm != kNoJob32) best = min(best, ((unsigned long long)jb << 32) | (unsigned long long)pm);
            }
            best = wave_min_u64(best);
            if (lane == 0 && best != ~0ull) atomicMin(&s_best, best);
            __syncthreads();
            const unsigned long long b = s_best;
            if (b != ~0ull) { found = true; ji = (uint32_t)(b >> 32); jk = (uint32_t)b; }
        }
        if (!found) {
            // (k0, the lowest later critical job that reaches V with it)
            const int k0pos = min((int)w.pos[k0job], P - 1);
            uint32_t sh, klo, span;
            const bool ok = key_range(sc, w.seg_grp[k0pos >> 6], sh, klo, span);
            const uint32_t xk = w.cu[k0pos] - sh;
            uint32_t best = kNoJob32;
            for (int p = sc.sbase + tid; p < sc.send; p += kSelBlock) {
                const uint32_t jb = w.job[p];
                if (ok && jb != kNoJob32 && jb > k0job && __usad(w.cu[p], xk, 0u) - klo <= span) best = min(best, jb);
            }
            best = wave_min_u32(best);
            if (lane == 0 && best != kNoJob32) atomicMin(&s_later, best);
            __syncthreads();
            ji = k0job;
            jk = s_later;
        }
        if (tid == 0) {
            // (independent loads first: one thread, every dependent round trip to memory counts)
            const bool valid = ji < (uint32_t)N && jk < (uint32_t)N && ji < jk;
            const int passes = ctrl->passes;
            const int pi = valid ? min((int)w.pos[ji], P - 1) : 0, pk = valid ? min((int)w.pos[jk], P - 1) : 0;
            const uint32_t at_pi = w.job[pi], at_pk = w.job[pk], xi = w.cu[pi], xk = w.cu[pk];
            const int ga = w.seg_grp[pi >> 6], gb = w.seg_grp[pk >> 6];
            if (!valid || at_pi != ji || at_pk != jk) {
                ctrl->status = MMBP_ST_INTERNAL; ctrl->stop = 1;
            } else {
                const long long d = (long long)((xi - kBias) >> 1) - (long long)((xk - kBias) >> 1);
                w.load[ga] = (long long)s_ld[ga] - d;     // the loads of this path fit 32 bits: s_ld holds them exactly
                w.load[gb] = (long long)s_ld[gb] + d;
                w.cu[pi] = xk; w.cu[pk] = xi;
                w.job[pi] = jk; w.job[pk] = ji;
                w.pos[ji] = (uint32_t)pk; w.pos[jk] = (uint32_t)pi;
                asg[ji] = gb; asg[jk] = ga;
                if (o.applied_log)
                    o.applied_log[(size_t)s * max_passes + passes] =
                        (uint64_t)N * (uint64_t)M + (uint64_t)ji * (uint64_t)N + (uint64_t)jk;
                ctrl->passes = passes + 1;
            }
        }
    }
    __syncthreads();
    g_prep_pass(w, o, s, M, max_passes, last_launch != 0, true, &s_ntask);
}

}  // namespace

size_t ls_grid_workspace_bytes(int S, int N, int M) { return (size_t)S * grid_layout(N, M).total; }

int ls_grid_pass_limit() { return kMaxPassLaunches; }

hipError_t launch_ls_grid(const void *cost, int dtype, int S, int N, int M, int cap, int max_passes, int prune,
                          int32_t *assign, int64_t *load_out, int64_t *makespan_out, int32_t *passes_out,
                          uint64_t *evals_out, uint64_t *applied_log, int32_t *status_out, void *workspace,
                          hipStream_t st)
{
    OutPtrs o{load_out, makespan_out, passes_out, status_out, evals_out, applied_log};
    // Tasks are row blocks of 1024 x column chunks.  With few clients there are few client pairs:
    // the chunk shrinks until a pass has about a thousand tasks (estimated for balanced clients),
    // and the evaluation gets no more workgroups than it can use.
    const long long avg = (N + M - 1) / M, pairs = prune ? (long long)(M - 1) : (long long)M * (M - 1) / 2;
    auto est_tasks = [&](int chunk) { return pairs * ((avg + 1023) / 1024) * ((avg + chunk - 1) / chunk); };
    int cchunk = kColChunk;
    while (cchunk > kMinColChunk && est_tasks(cchunk) < 1024) cchunk >>= 1;
    const long long want = est_tasks(cchunk) * 3 / 2 + M;
    const int egrid = want < 64 ? 64 : want < kEvalGrid ? (int)want : kEvalGrid;
    if (dtype == MMBP_I32)
        grid_stage_kernel<int32_t><<<dim3(S), dim3(kSelBlock), 0, st>>>((const int32_t *)cost, N, M, cap, max_passes,
                                                                       prune, cchunk, egrid, assign, o, workspace);
    else
        grid_stage_kernel<int64_t><<<dim3(S), dim3(kSelBlock), 0, st>>>((const int64_t *)cost, N, M, cap, max_passes,
                                                                       prune, cchunk, egrid, assign, o, workspace);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int launches = max_passes < kMaxPassLaunches ? max_passes : kMaxPassLaunches;
    const int has_flag = grid_has_flag(N, M) ? 1 : 0;
    for (int i = 0; i < launches; i++) {
        grid_eval_kernel<<<dim3(egrid, S), dim3(kEvalBlock), 0, st>>>(N, M, workspace);
        if (has_flag) grid_flag_kernel<<<dim3(kFlagGrid, S), dim3(kFlagBlock), 0, st>>>(N, M, workspace);
        const int last = (i == launches - 1 && launches < max_passes) ? 1 : 0;
        if (dtype == MMBP_I32)
            grid_select_kernel<int32_t><<<dim3(S), dim3(kSelBlock), 0, st>>>((const int32_t *)cost, N, M, cap, max_passes,
                                                                            assign, o, workspace, last, has_flag);
        else
            grid_select_kernel<int64_t><<<dim3(S), dim3(kSelBlock), 0, st>>>((const int64_t *)cost, N, M, cap, max_passes,
                                                                            assign, o, workspace, last, has_flag);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace mmbp
