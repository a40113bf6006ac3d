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
// (v_sad_u32 would fuse them but issues at quarter rate).
//
// Tasks.  Every unordered client pair is evaluated once per pass.  A table built with the layout
// lists the tasks (row unit of client g: up to 4 segments of 64 rows) x (chunk of up to kChunk
// columns of a client b > g), and per row unit / column chunk there is a record of its own.
//
// A pass has three phases.  The makespan can only fall if load leaves the client with the largest
// load ("critical"), so phase A evaluates what involves it: its moves, and its swap tiles, always
// (row unit of another client) x (column chunk of the critical client), a contiguous range per
// wave.  Wave 0 waits for the other waves' minima on a counter and selects the candidate while all
// waves (wave 0 too, when it is done) evaluate the rest of the scan in phase C: the tasks of the
// table that do not involve the critical client and the moves of the other clients, dealt out one
// at a time from an LDS counter.  Those candidates keep the critical load, so their makespan is at
// least the current one and cannot change the decision; their minimum is kept and checked against
// that bound.  Nothing is changed before the barrier that ends phase C; then wave 0 applies the
// candidate and opens the next pass while the other waves put the row minima back.
//
// Exact lowest-id tie-break without a second full scan.  Phase A min-combines, per non-critical
// job, its best makespan against the critical client (rowkey) and tracks the smallest (makespan,
// job) of those.  Wave 0 then knows the best value V and k0 = the lowest-index non-critical job of a
// best swap; only critical jobs with a lower index than k0 ("early") can carry a lower id: they are
// taken in index order, four at a time, against the flagged jobs (rowkey == V); k0's own partners
// are scanned; the packed minimum (i, k, pos_i, pos_k) is applied.  In the full scan moves are
// value-only in phase A and rescanned for the id when a move wins.
//
// Pruned scan (PRUNE): only the candidates that involve the critical client are looked at (the others
// cannot lower max_j t_j).  The positions of every client are then kept in ascending order of cu
// (sorted after each regrouping: one wave per client where no range exceeds 64 positions, a bitonic
// network over the layout otherwise; a swap or a move removes one entry and inserts the other in place).
// Its ranges are multiples of 16 positions, not 64, with a few free positions for moves to enter in place, so
// several small clients share a 64-position segment and the rows' client and load are per lane.
// A row's best partner in the critical client is found by binary search: the nearest column at or
// above x and the nearest below it, i.e. the same key min |y - x| the tile computes, in O(log n)
// per row instead of one subtraction per column; where that client holds at most kPruneTileCols jobs
// the rows run the tile arithmetic against all of them instead (no chain of dependent LDS reads).
// The moves off the critical client are evaluated with their ids by all waves (a slice of the target
// clients each), so a winning move needs no second look.  Selection, tie-break and apply are shared.
//
// Exactness: all loads stay at or below the initial makespan T0; with T0 + 2*max T_i < 2^29 every
// quantity above is exact in 32 bits: x lies in (2^29, 3*2^29), a real |y - x| is below 2^29, a
// wrapped difference is above 7*2^29, and an empty column (cu = 6*2^29) gives d in (3*2^29, 5*2^29),
// which can win neither the minimum nor (negated) the maximum against a real column.  Scenarios
// that do not satisfy the bound stay pending for the 64-bit kernel.
//
// Termination by construction: every loop of a pass is bounded by N, M and the padded size, every
// barrier is reached under conditions read from LDS after a barrier, the pass loop is capped, the
// one in-workgroup wait (wave 0 on the other waves' posts, which never depend on wave 0) has a spin
// limit, and states that cannot occur stop the scenario with MMBP_ST_INTERNAL instead of being
// acted on.
#include "mmbp_dev.hpp"
#include "ls_tile.hpp"

namespace mmbp {
namespace {

#ifndef MMBP_LDS_CHUNK
#define MMBP_LDS_CHUNK 256
#endif
#ifndef MMBP_LDS_WPE
#define MMBP_LDS_WPE 4
#endif
constexpr int kChunk = MMBP_LDS_CHUNK;         // columns per task (multiple of 64, at most 256)
constexpr int kSpinLimit = 1 << 20;            // bound of the one in-workgroup wait (far above any real wait)
constexpr size_t kLdsLimit = 156 * 1024;       // a CU has 160 KB, all of which one workgroup may use; above 64 KB the
                                               // launch raises the kernel's dynamic-LDS attribute first
static_assert(kChunk % 64 == 0 && kChunk <= 64 * kRMax, "a chunk must be runnable as the row side of a tile");

struct Ctrl {
    unsigned long long pairs_per_scan;
    unsigned long long k0key;     // min over the rows against the critical client of (makespan << 32 | job << 16 | pos)
    uint32_t counted;             // candidates the waves have evaluated in this scan (sum of their own counts)
    unsigned long long wsum[16];
    unsigned long long wmax[16];
    long long T0;
    uint32_t vswap, vmove, vrest;  // per-pass minima: swaps and moves that involve the critical client, the rest
    int nfeas, P, rebuild, ntask, nchunk;
    int next;                     // work counter of the rest of the scan
    int adone;                    // waves that have posted their phase-A minima
    Top3 top;                     // three largest loads and their clients, published by wave 0
    int stop;
    int bad_cost, bad_assign;
    unsigned long long kmove;     // min over the moves off the critical client of (makespan << 32 | move id)
};

struct Lds {
    uint32_t *cu, *rowkey;        // rowkey[p]: best swap makespan of the job at p against the critical client
    uint16_t *rowkey16;           // the pruned scan keeps the low 16 bits of it (same memory, half of it): a filter for the
                                  // rows that may attain the best value; every use re-checks the value exactly
    uint16_t *job;
    unsigned long long *tasks;    // row unit record | chunk record << 32
    uint32_t *chunks;             // c0/64 | columns (jobs of the client in the chunk) << 10 | b << 19
    uint32_t *uinfo;              // per row unit: rowbase/64 | R << 10 | g << 13 | rows (jobs of the client in the unit) << 21
    long long *load;
    int *cnt, *gstart, *fillc, *feas, *chpre, *upre;
    uint32_t *tdl, *tr1;          // per client, for the selection: l_g - l_critical and the key bound of a best swap
    uint8_t *seg_grp;
    Ctrl *ctrl;
};

__host__ __device__ inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

constexpr int kPruneGranShift = 4, kPruneGran = 1 << kPruneGranShift;   // positions a client's range is a multiple of (pruned layout)
constexpr int kPruneSlack = 4;                                          // free positions every client gets when the jobs are regrouped

struct LdsDims {
    size_t P, U, C, T;            // padded positions, row units, column chunks, tasks (upper bounds)
};
__host__ __device__ inline LdsDims lds_dims(int N, int M, bool prune)
{
    LdsDims d;
    // multiple of 64: keeps every array 16-byte aligned.  The full scan's clients own whole 64-position segments (a
    // tile's rows are one client's); the pruned scan's own multiples of kPruneGran positions with at least
    // kPruneSlack of them free after a regrouping (moves then enter in place), so small clients share a segment.
    d.P = prune ? ((size_t)N + (size_t)(kPruneSlack + kPruneGran - 1) * (size_t)M + 63u) / 64u * 64u
                : ((size_t)N + 63u) / 64u * 64u + 64u * (size_t)M;
    d.U = prune ? 0 : d.P / (64u * kRMax) + (size_t)M;       // the pruned scan searches sorted columns: no tile tables
    d.C = prune ? 0 : (size_t)N / kChunk + (size_t)M;
    d.T = d.U * d.C;
    return d;
}

__host__ __device__ inline size_t lds_bytes(int N, int M, bool prune)
{
    const LdsDims d = lds_dims(N, M, prune);
    size_t b = 0;
    b += 4 * d.P;                     // cu
    b += (prune ? 2 : 4) * d.P;       // rowkey (16 bits per row in the pruned scan)
    b += 2 * d.P;                     // job
    b = align_up(b, 16);
    b += 8 * d.T;                     // tasks
    b += 4 * d.C;                     // chunks
    b += 4 * d.U;                     // uinfo
    b = align_up(b, 16);
    b += 8 * (size_t)M;               // load
    b += 4 * (size_t)(M + 1) * 8;     // cnt, gstart, fillc, feas, chpre, upre, tdl, tr1
    b += align_up(d.P / kPruneGran + 1, 16);  // seg_grp (one entry per 64 positions in the full scan, per kPruneGran in the pruned scan)
    b = align_up(b, 16);
    b += sizeof(Ctrl);
    return b;
}

__device__ inline Lds carve(unsigned char *base, int N, int M, bool prune)
{
    const LdsDims d = lds_dims(N, M, prune);
    Lds l;
    size_t o = 0;
    l.cu = (uint32_t *)(base + o); o += 4 * d.P;
    l.rowkey = (uint32_t *)(base + o); l.rowkey16 = (uint16_t *)(base + o); o += (prune ? 2 : 4) * d.P;
    l.job = (uint16_t *)(base + o); o += 2 * d.P;
    o = align_up(o, 16);
    l.tasks = (unsigned long long *)(base + o); o += 8 * d.T;
    l.chunks = (uint32_t *)(base + o); o += 4 * d.C;
    l.uinfo = (uint32_t *)(base + o); o += 4 * d.U;
    o = align_up(o, 16);
    l.load = (long long *)(base + o); o += 8 * (size_t)M;
    l.cnt = (int *)(base + o); o += 4 * (size_t)(M + 1);
    l.gstart = (int *)(base + o); o += 4 * (size_t)(M + 1);
    l.fillc = (int *)(base + o); o += 4 * (size_t)(M + 1);
    l.feas = (int *)(base + o); o += 4 * (size_t)(M + 1);
    l.chpre = (int *)(base + o); o += 4 * (size_t)(M + 1);
    l.upre = (int *)(base + o); o += 4 * (size_t)(M + 1);
    l.tdl = (uint32_t *)(base + o); o += 4 * (size_t)(M + 1);
    l.tr1 = (uint32_t *)(base + o); o += 4 * (size_t)(M + 1);
    l.seg_grp = (uint8_t *)(base + o); o += align_up(d.P / kPruneGran + 1, 16);
    o = align_up(o, 16);
    l.ctrl = (Ctrl *)(base + o);
    return l;
}

// three largest loads with their clients for M <= 64 (one load per lane): three wave maxima, each
// taking the lowest client among equal loads and leaving it out of the next
__device__ __forceinline__ Top3 wave_top3_small(uint32_t vload, int M, int lane)
{
    bool in = lane < M;
    auto next = [&](uint32_t &v, int &jout) {
        const uint32_t mx = wave_max_u32(in ? vload : 0u);
        const unsigned long long m = __ballot(in && vload == mx);
        jout = m ? (int)__builtin_ctzll(m) : -1;
        v = m ? mx : 0u;
        if (lane == jout) in = false;
    };
    Top3 t;
    next(t.v0, t.j0);
    next(t.v1, t.j1);
    next(t.v2, t.j2);
    return t;
}

// One tile: rows = R segments at rowbase (client X, load lx), columns [c0, c1) (client Y, load ly).
// star: Y is the critical client -> the rows' best makespans go to rowkey and to the (makespan,
// job, pos) minimum kbest.
template <int R>
__device__ __forceinline__ void run_tile(const Lds &l, int rowbase, int c0, int c1, uint32_t lx, uint32_t ly,
                                         uint32_t oth, bool star, int lane, uint32_t &sbest, unsigned long long &kbest)
{
    uint32_t rowx[R], x[R], key[R];
#pragma unroll
    for (int r = 0; r < R; r++) {
        rowx[r] = l.cu[rowbase + 64 * r + lane];
        x[r] = rowx[r] - (lx - ly);
    }
    tile_columns<R>(l.cu, x, c0, c1, key);
    if (!star) {
        // only the tile's best makespan is wanted, and the makespan grows with the key: one conversion
        // for the smallest key of the lane's rows (an empty row's key is out of range and converts to none)
        uint32_t kmin = kInf;
#pragma unroll
        for (int r = 0; r < R; r++) kmin = min(kmin, rowx[r] != kPad ? key[r] : kInf);
        sbest = min(sbest, swap_value(kmin, lx + ly, oth));
        return;
    }
#pragma unroll
    for (int r = 0; r < R; r++) {
        const uint32_t v = rowx[r] != kPad ? swap_value(key[r], lx + ly, oth) : kInf;
        sbest = min(sbest, v);
        if (v != kInf) {
            const int p = rowbase + 64 * r + lane;
            atomicMin(&l.rowkey[p], v);
            kbest = min(kbest, ((unsigned long long)v << 32) | ((unsigned long long)l.job[p] << 16) | (unsigned long long)p);
        }
    }
}

// Sorts the positions of every client by cu, ascending (all threads; barriers inside).  A bitonic
// network whose comparators all put the smaller entry at the lower position, so positions beyond P
// act as +infinity without being stored; entries of different clients never change order (clients
// occupy ascending position ranges), empty positions (kPad) end up last in their client's range.
template <int BLOCK>
__device__ void sort_groups(const Lds &l, int P, int M)
{
    const int tid = threadIdx.x;
    int maxcnt = 0;                                      // jobs of the largest client (every thread reads all counts: broadcasts)
    for (int g = 0; g < M; g++) maxcnt = max(maxcnt, l.cnt[g]);
    if (maxcnt + kPruneSlack <= kWave) {                 // (a range is its jobs plus at most the slack, rounded up: at most 64 positions)
        // No client's range has more positions than a wave has lanes: a wave sorts a client's range in
        // its registers (21 compare-exchange steps across the lanes) instead of all threads running the network
        // over the whole layout (about a hundred steps with a barrier each, most of them over empty positions
        // when clients are many and small).
        const int lane = tid & 63;
        for (int g = tid >> 6; g < M; g += BLOCK / kWave) {
            const int base = min(max(l.gstart[g], 0), P), slots = min(max(l.gstart[g + 1], base), P) - base;
            const bool in = lane < slots;
            uint32_t x = in ? l.cu[base + lane] : kPad, jb = in ? (uint32_t)l.job[base + lane] : (uint32_t)kNoJob;
            for (int k = 2; k <= kWave; k <<= 1)
                for (int j = k >> 1; j > 0; j >>= 1) {
                    const uint32_t px = (uint32_t)__shfl_xor((int)x, j), pj = (uint32_t)__shfl_xor((int)jb, j);
                    const bool take_min = ((lane & j) == 0) == ((lane & k) == 0);      // ascending blocks: the lower lane keeps the smaller
                    const bool sw = take_min ? px < x : px > x;                        // (equal keys: both lanes keep their own)
                    x = sw ? px : x;
                    jb = sw ? pj : jb;
                }
            if (in) { l.cu[base + lane] = x; l.job[base + lane] = (uint16_t)jb; }     // (empty positions sort last: they stay where they were)
        }
        __syncthreads();
        return;
    }
    int P2 = 1;
    while (P2 < P) P2 <<= 1;
    for (int k = 2; k <= P2; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int t = tid; t < (P2 >> 1); t += BLOCK) {
                const int blk = t / j, off = t - blk * j;
                int i, q;
                if (j == (k >> 1)) { i = blk * k + off; q = blk * k + (k - 1 - off); }
                else { i = blk * 2 * j + off; q = i + j; }
                if (q < P && l.seg_grp[i >> kPruneGranShift] == l.seg_grp[q >> kPruneGranShift]) {
                    const uint32_t a = l.cu[i], b = l.cu[q];
                    if (a > b) {
                        l.cu[i] = b; l.cu[q] = a;
                        const uint16_t ja = l.job[i];
                        l.job[i] = l.job[q]; l.job[q] = ja;
                    }
                }
            }
            __syncthreads();
        }
}

constexpr int kPruneRows = 2;              // row segments per lane in that tile
constexpr int kPruneTileCols = 40;         // the pruned scan takes the tile arithmetic, not the binary search, up to this many columns

// min over the n sorted entries cu[sb .. sb+n) of |cu - x|: the nearest at or above x, the nearest below
__device__ __forceinline__ uint32_t nearest_sorted(const uint32_t *cu, int sb, int n, uint32_t x)
{
    int lo = 0, hi = n;                                  // first entry >= x
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (cu[sb + mid] < x) lo = mid + 1; else hi = mid;
    }
    const uint32_t up = lo < n ? cu[sb + lo] - x : kInf;
    const uint32_t dn = lo > 0 ? x - cu[sb + lo - 1] : kInf;
    return min(up, dn);
}

// The pruned layout's starts (no tile tables): a prefix sum of the clients' slot counts, 64 clients per step of
// one wave (a serial walk over the clients is a chain of dependent LDS accesses: with 200 clients it was most
// of the staging of a small scenario).  Out of line: it runs once per regrouping, and inlined it raised the
// register pressure of the pass loop.
__device__ __attribute__((noinline)) void sorted_layout_starts(const Lds &l, int N, int M, int cap, int plimit, int lane)
{
    int running = 0, nf = 0;
    unsigned long long sq = 0;
    for (int j0 = 0; j0 < M; j0 += kWave) {
        const int j = j0 + lane;
        const int n = j < M ? min(max(l.cnt[j], 0), N) : 0;
        const int room = j < M ? min(max(cap - n, 0), kPruneSlack) : 0;      // (a client never holds more than cap jobs)
        const int slots = ((n + room + kPruneGran - 1) >> kPruneGranShift) * kPruneGran;
        int incl = slots;
        for (int off = 1; off < kWave; off <<= 1) {
            const int up = __shfl_up(incl, off);
            if (lane >= off) incl += up;
        }
        const int start = min(running + incl - slots, plimit);
        const int end = min(start + slots, plimit);
        if (j < M) {
            l.gstart[j] = start;
            l.chpre[j] = 0; l.upre[j] = 0;
            for (int q = start >> kPruneGranShift; q < (end >> kPruneGranShift); q++) l.seg_grp[q] = (uint8_t)j;
        }
        running += __builtin_amdgcn_readlane(incl, kWave - 1);
        const bool ok = j < M && n < cap;         // move targets, ascending
        const unsigned long long m = __ballot(ok);
        if (ok) l.feas[nf + __popcll(m & ((1ull << lane) - 1ull))] = j;
        nf += __popcll(m);
        sq += (unsigned long long)n * (unsigned long long)n;
    }
    for (int off = 32; off >= 1; off >>= 1) sq += __shfl_xor(sq, off);
    if (lane == 0) {
        const int pos = min(running, plimit);
        l.gstart[M] = pos;
        l.chpre[M] = 0; l.upre[M] = 0;
        const int pend = min((pos + 63) & ~63, plimit);  // the layout ends on a whole segment: empty positions after the last client
        for (int q = pos >> kPruneGranShift; q < (pend >> kPruneGranShift); q++) l.seg_grp[q] = 0;
        l.ctrl->P = pend;
        l.ctrl->nfeas = nf;
        l.ctrl->nchunk = 0;
        l.ctrl->ntask = 0;
        l.ctrl->pairs_per_scan = ((unsigned long long)N * (unsigned long long)N - sq) / 2ull;
    }
}

// Groups the jobs by client and builds the chunk and task tables (all threads; barriers inside).
template <typename CostT, int BLOCK>
__device__ void build_layout(const Lds &l, const CostT *__restrict__ c, const int32_t *asg, int N, int M, int cap, bool sorted)
{
    const int tid = threadIdx.x;
    const LdsDims d = lds_dims(N, M, sorted);            // (sorted = the pruned scan: its tables have no entries)
    if (sorted) {
        if (tid < kWave) sorted_layout_starts(l, N, M, cap, (int)d.P, tid);
    } else if (tid == 0) {
        int pos = 0, nf = 0, nch = 0, nu = 0;
        unsigned long long sq = 0;
        for (int g = 0; g < M; g++) {
            l.gstart[g] = pos;
            l.chpre[g] = min(nch, (int)d.C);
            l.upre[g] = min(nu, (int)d.U);
            const int n = l.cnt[g];
            const int ns = min((n + 63) >> 6, (int)((d.P - pos) >> 6));
            for (int q = 0; q < ns; q++) l.seg_grp[(pos >> 6) + q] = (uint8_t)g;
            pos += ns * 64;
            nch += (n + kChunk - 1) / kChunk;
            nu += (ns + kRMax - 1) / kRMax;
            if (n < cap) l.feas[nf++] = g;
            sq += (unsigned long long)n * (unsigned long long)n;
        }
        l.gstart[M] = pos;
        l.chpre[M] = min(nch, (int)d.C);
        l.upre[M] = min(nu, (int)d.U);
        l.ctrl->P = pos;
        l.ctrl->nfeas = nf;
        l.ctrl->nchunk = min(nch, (int)d.C);
        l.ctrl->ntask = 0;
        l.ctrl->pairs_per_scan = ((unsigned long long)N * (unsigned long long)N - sq) / 2ull;
    }
    for (int j = tid; j < M; j += BLOCK) l.fillc[j] = 0;
    __syncthreads();
    const int P = l.ctrl->P;
    for (int p = tid; p < P; p += BLOCK) {
        l.cu[p] = kPad; l.job[p] = kNoJob;
        if (sorted) l.rowkey16[p] = 0xFFFFu; else l.rowkey[p] = kInf;
    }
    // chunk records: one thread per client
    for (int g = tid; g < M; g += BLOCK) {
        const int n = l.cnt[g];
        for (int k = l.chpre[g], q = 0; k < l.chpre[g + 1]; k++, q++)
            l.chunks[k] = (uint32_t)((l.gstart[g] + q * kChunk) >> 6) | ((uint32_t)min(kChunk, n - q * kChunk) << 10) |
                          ((uint32_t)g << 19);
    }
    __syncthreads();
    for (int i = tid; i < N; i += BLOCK) {
        const int a = asg[i];
        const int p = l.gstart[a] + atomicAdd(&l.fillc[a], 1);
        l.cu[p] = 2u * (uint32_t)c[i] + kBias;
        l.job[p] = (uint16_t)i;
    }
    // task records: one thread per row unit; its tasks (all chunks of later clients) are contiguous
    const int nU = l.upre[M], nCh = l.ctrl->nchunk;
    for (int u = tid; u < nU; u += BLOCK) {
        int g = 0;
        while (g + 1 < M && l.upre[g + 1] <= u) g++;
        const int blk = (u - l.upre[g]) * kRMax;
        const int gseg = (l.gstart[g + 1] - l.gstart[g]) >> 6;
        const uint32_t w0 = (uint32_t)((l.gstart[g] >> 6) + blk) | ((uint32_t)min(kRMax, gseg - blk) << 10) | ((uint32_t)g << 13) |
                            ((uint32_t)min(64 * kRMax, max(l.cnt[g] - blk * 64, 0)) << 21);
        if (u < (int)d.U) l.uinfo[u] = w0;
        const int k0 = l.chpre[g + 1], n = nCh - k0;
        if (n <= 0) continue;
        const int base = atomicAdd(&l.ctrl->ntask, n);
        if (base + n > (int)d.T) continue;               // cannot happen: T bounds the table
        for (int q = 0; q < n; q++) l.tasks[base + q] = (unsigned long long)w0 | ((unsigned long long)l.chunks[k0 + q] << 32);
    }
    __syncthreads();
    if (sorted) sort_groups<BLOCK>(l, min(l.ctrl->P, (int)d.P) & ~63, M);
}

template <typename CostT, int BLOCK, bool SMALLM, bool PRUNE>
__global__ __launch_bounds__(BLOCK, PRUNE ? 6 : MMBP_LDS_WPE) void ls_lds_kernel(
    const CostT *__restrict__ cost_all, int N, int M, int cap, int max_passes, int32_t *assign_all,
    int64_t *load_out, int64_t *makespan_out, int32_t *passes_out, uint64_t *evals_out,
    uint64_t *applied_log, int32_t *status_out)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const Lds l = carve(lds_raw, N, M, PRUNE);
    Ctrl *ctrl = l.ctrl;
    const int s = blockIdx.x;
    const CostT *c = cost_all + (size_t)s * N;
    int32_t *asg = assign_all + (size_t)s * N;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int kWaves = BLOCK / kWave;
    constexpr int kGrpShift = PRUNE ? kPruneGranShift : 6;   // positions per entry of seg_grp

    // ---------------- stage: validation, counts, loads ----------------
    for (int j = tid; j < M; j += BLOCK) { l.load[j] = 0; l.cnt[j] = 0; }
    if (tid == 0) {
        ctrl->bad_cost = 0; ctrl->bad_assign = 0; ctrl->stop = 0; ctrl->rebuild = 0;
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
    build_layout<CostT, BLOCK>(l, c, asg, N, M, cap, PRUNE);

    // loads stay below 2^29 on this path: their low words are used
    auto load32 = [&](int g) -> uint32_t { return (uint32_t)l.load[g]; };
    const int Pmax = N + 64 * M;
    const int Tmax = (int)lds_dims(N, M, PRUNE).T, Umax = (int)lds_dims(N, M, PRUNE).U, Cmax = (int)lds_dims(N, M, PRUNE).C;
    // A workgroup's waves go round the four SIMDs of its CU; the two halves of a SIMD's waves get
    // neighbouring ranges of the task table, so the SIMDs carry equal shares when waves outnumber them.
    const int twave = kWaves >= 8 ? (wave & 3) * (kWaves / 4) + (wave >> 2) : wave;

    // Pass accounting lives in wave 0's registers (uniform); LDS only carries what the other
    // waves read: the stop and rebuild flags, the three largest loads, the per-pass minima.
    int w_passes = 0, w_iters = 0, w_status = MMBP_ST_OK;
    bool w_stop = false;
    unsigned long long w_evals = 0, w_pairs = ctrl->pairs_per_scan;

    // Opens a pass (wave 0 only, all 64 lanes): accounting, the three largest loads for everybody,
    // the per-pass minima and the row minima back to "none".  vnew: lane j holds the load of
    // client j (SMALLM only; otherwise the loads are read back from LDS).
    auto open_pass = [&](uint32_t vnew, bool reset_rows) {
        w_iters += 1;
        if ((long long)w_iters > (long long)max_passes + 1) { w_status = MMBP_ST_INTERNAL; w_stop = true; }
        else if (w_stop) { }
        else if (w_passes == max_passes) { w_status = MMBP_ST_TRUNCATED; w_stop = true; }
        __builtin_amdgcn_wave_barrier();   // lanes of a wave run in lockstep: earlier LDS updates are complete
        const Top3 t = SMALLM ? wave_top3_small(vnew, M, lane) : wave_top3(l.load, M, lane);
        if (lane == 0) {
            ctrl->top = t;
            ctrl->vswap = kInf; ctrl->vmove = kInf; ctrl->vrest = kInf; ctrl->k0key = ~0ull;
            if constexpr (PRUNE) ctrl->kmove = ~0ull;
            ctrl->next = 0; ctrl->adone = 0; ctrl->counted = 0;
            if (w_stop) ctrl->stop = 1;
        }
        if (reset_rows) {
            const int P = min(ctrl->P, Pmax) & ~63;
            uint4 *rk = reinterpret_cast<uint4 *>(l.rowkey);
            for (int q = lane; q < (P >> (PRUNE ? 3 : 2)); q += kWave) rk[q] = make_uint4(kInf, kInf, kInf, kInf);
        }
    };
    if (wave == 0) open_pass(SMALLM ? (lane < M ? load32(lane) : 0u) : 0u, true);   // (build_layout ended with a barrier)

    // ---------------- pass loop ----------------
    // A pass has three phases.  A: the candidates that can lower the makespan (they take load off
    // the critical client): its moves and its swap tiles, all waves; barrier B1.  B: wave 0 selects
    // the candidate to apply, changing nothing yet.  C: the rest of the scan (candidates that leave
    // the critical client alone: their makespan is at least the current one, so they cannot change
    // the decision), dealt out tile by tile from a counter to all waves, wave 0 joining when its
    // selection is done; barrier B2.  Then wave 0 applies the candidate and opens the next pass.
    enum { kActNone = 0, kActStop, kActMove, kActSwap, kActError };
    for (;;) {
        __syncthreads();                                 // B0: layout, loads, top-3 and flags are published
        if (ctrl->stop) break;
        if (ctrl->rebuild) {                             // a move was applied: regroup the jobs
            build_layout<CostT, BLOCK>(l, c, asg, N, M, cap, PRUNE);
            if (tid == 0) ctrl->rebuild = 0;             // (after the last barrier of build_layout: nobody
                                                         //  reads the flag before the next B0)
            w_pairs = ctrl->pairs_per_scan;              // the pair count of the scan that starts now
        }

        const int P = min(ctrl->P, Pmax) & ~63;
        const int nseg = P >> 6;
        const int nfeas = min(ctrl->nfeas, M);
        const int ntask = min(ctrl->ntask, Tmax);
        Top3 top;
        top.v0 = uniu(ctrl->top.v0); top.v1 = uniu(ctrl->top.v1); top.v2 = uniu(ctrl->top.v2);
        top.j0 = uni(ctrl->top.j0); top.j1 = uni(ctrl->top.j1); top.j2 = uni(ctrl->top.j2);
        const uint32_t T = top.v0;
        const int astar = min(max(top.j0, 0), M - 1);
        const uint32_t vload = SMALLM ? (lane < M ? load32(lane) : 0u) : 0u;   // one load per lane
        auto wload = [&](int g) -> uint32_t {
            return SMALLM ? (uint32_t)__builtin_amdgcn_readlane((int)vload, g) : uniu(load32(g));
        };
        uint32_t w_cnt = 0;                              // candidates this wave evaluates in this scan (uniform; a scan of a
                                                         // layout that fits the LDS has far fewer than 2^32)
        // w0: row unit record, w1: chunk record (their client fields are passed decoded as X and Y)
        auto run = [&](uint32_t w0, int X, uint32_t w1, int Y, bool star, uint32_t &sb, unsigned long long &kb) {
            const int rowbase = (int)(w0 & 0x3FFu) << 6, R = (int)((w0 >> 10) & 7u), c0 = (int)(w1 & 0x3FFu) << 6;
            const int ncols = (int)((w1 >> 10) & 0x1FFu), c1 = c0 + ((ncols + 7) & ~7);
            if (R < 1 || R > kRMax || c1 <= c0 || c1 > Pmax || rowbase + 64 * R > Pmax) return;   // cannot happen
            w_cnt += ((w0 >> 21) & 0x1FFu) * (uint32_t)ncols;   // jobs in the unit x jobs in the chunk
            const uint32_t lx = wload(X), ly = wload(Y);
            const uint32_t oth = others_max(top, X, Y);
            if (R == 1) run_tile<1>(l, rowbase, c0, c1, lx, ly, oth, star, lane, sb, kb);
            else if (R == 2) run_tile<2>(l, rowbase, c0, c1, lx, ly, oth, star, lane, sb, kb);
            else if constexpr (kRMax >= 3) {
                if (R == 3) run_tile<3>(l, rowbase, c0, c1, lx, ly, oth, star, lane, sb, kb);
                else run_tile<kRMax>(l, rowbase, c0, c1, lx, ly, oth, star, lane, sb, kb);
            }
        };
        auto segment_moves = [&](int seg, int g) -> uint32_t {     // best move makespan of the 64 positions of a segment
                const uint32_t x = l.cu[seg * 64 + lane];
                w_cnt += (uint32_t)__popcll(__ballot(x != kPad)) * (uint32_t)(M - 1);
                const uint32_t ci = (x - kBias) >> 1;
                const uint32_t la = load32(g);
                uint32_t m = kInf;
                for (int q = 0; q < nfeas; q++) {
                    const int b = l.feas[q];
                    if (b == g) continue;
                    const uint32_t v = max(max(la - ci, load32(b) + ci), others_max(top, g, b));
                    m = min(m, v);
                }
            return x != kPad ? m : kInf;
        };

        // ---- phase A: moves off the critical client, swap tiles (row unit of another client) x
        //      (column chunk of the critical client); each wave a contiguous range of them ----
        uint32_t mbest = kInf, sbest = kInf;
        unsigned long long kbest = ~0ull;
        const int sega = min(max(uni(l.gstart[astar]), 0), P) >> 6, segb = min(max(uni(l.gstart[astar + 1]), 0), P) >> 6;
        if constexpr (!PRUNE) {
            if (nfeas > 0)
                for (int seg = sega + wave; seg < segb; seg += kWaves) mbest = min(mbest, segment_moves(seg, astar));
        }
        if constexpr (PRUNE) {
            // every position outside the critical client against its sorted columns
            const int sb = min(max(uni(l.gstart[astar]), 0), P), sn = min(max(uni(l.cnt[astar]), 0), P - sb);
            const int s1 = min(max(uni(l.gstart[astar + 1]), 0), P);
            const uint32_t lstar = wload(astar);
            if (sn > 0 && sn <= kPruneTileCols) {
                // Few columns: the tile arithmetic against all of them (two vector instructions per candidate, the
                // columns read as broadcasts that do not depend on the rows) is shorter than a binary search per
                // row, which is a chain of dependent LDS reads; two row segments per lane share the column reads
                // (four would spill under the pruned kernels' register limit).  A segment may hold several small
                // clients, so the client and its load are per lane.
                const int n4 = (sn + 3) >> 2;                  // (the positions after the last column are empty ones: no candidates)
                for (int base = wave; base < nseg; base += kPruneRows * kWaves) {
                    uint32_t x[kPruneRows], cx[kPruneRows], lsum[kPruneRows], oth[kPruneRows], key[kPruneRows];
#pragma unroll
                    for (int q = 0; q < kPruneRows; q++) {
                        const int seg = base + q * kWaves, pp = seg * 64 + lane;
                        const bool on = seg < nseg && (pp < sb || pp >= s1);      // (not the critical client's own positions)
                        const int g = on ? min((int)l.seg_grp[pp >> kPruneGranShift], M - 1) : 0;
                        const uint32_t lg = load32(g);
                        cx[q] = on ? l.cu[pp] : kPad;
                        x[q] = cx[q] - (lg - lstar);
                        lsum[q] = lg + lstar;
                        oth[q] = others_max(top, g, astar);
                    }
                    {
                        RowAcc acc[kPruneRows];
#pragma unroll
                        for (int q = 0; q < kPruneRows; q++) { acc[q].up = kInf; acc[q].mx = 0u; }
                        const uint4 *col = reinterpret_cast<const uint4 *>(l.cu + sb);
                        for (int k = 0; k < n4; k++) {
                            const uint4 c4 = col[k];
#pragma unroll
                            for (int q = 0; q < kPruneRows; q++) nearest_x4(acc[q], x[q], c4);
                        }
#pragma unroll
                        for (int q = 0; q < kPruneRows; q++) key[q] = nearest_key(acc[q]);
                    }
#pragma unroll
                    for (int q = 0; q < kPruneRows; q++) {
                        const int pp = (base + q * kWaves) * 64 + lane;
                        const uint32_t v = cx[q] != kPad ? swap_value(key[q], lsum[q], oth[q]) : kInf;
                        sbest = min(sbest, v);
                        if (v != kInf) {
                            l.rowkey16[pp] = (uint16_t)v;
                            kbest = min(kbest, ((unsigned long long)v << 32) | ((unsigned long long)l.job[pp] << 16) | (unsigned long long)pp);
                        }
                    }
                }
            } else if (sn > 0)
                for (int p = tid; p < P; p += BLOCK) {
                    if (p >= sb && p < s1) continue;
                    const uint32_t cx = l.cu[p];
                    if (cx == kPad) continue;
                    const int g = min((int)l.seg_grp[p >> kPruneGranShift], M - 1);
                    const uint32_t lg = load32(g);
                    const uint32_t v = swap_value(nearest_sorted(l.cu, sb, sn, cx - (lg - lstar)), lg + lstar, others_max(top, g, astar));
                    sbest = min(sbest, v);
                    if (v != kInf) {
                        l.rowkey16[p] = (uint16_t)v;     // one thread per row: nothing to combine
                        kbest = min(kbest, ((unsigned long long)v << 32) | ((unsigned long long)l.job[p] << 16) | (unsigned long long)p);
                    }
                }
        } else {
            const int nU = min(max(uni(l.upre[M]), 0), Umax);
            const int ua0 = min(max(uni(l.upre[astar]), 0), nU), nua = min(max(uni(l.upre[astar + 1]), 0), nU) - ua0;
            const int nCh = min(max(ctrl->nchunk, 0), Cmax);
            const int ca0 = min(max(uni(l.chpre[astar]), 0), nCh), nca = min(max(uni(l.chpre[astar + 1]), 0), nCh) - ca0;
            const int nstar = (nua >= 0 && nca > 0) ? (nU - nua) * nca : 0;
            const int lo = (int)(((long long)nstar * twave) / kWaves), hi = (int)(((long long)nstar * (twave + 1)) / kWaves);
            if (lo < hi) {
                int uq = lo / nca, cq = lo - uq * nca;
                for (int k = lo; k < hi; k++) {
                    const int u = uq < ua0 ? uq : uq + nua;
                    const uint32_t w0 = uniu(l.uinfo[min(u, Umax - 1)]), w1 = uniu(l.chunks[min(ca0 + cq, Cmax - 1)]);
                    run(w0, (int)((w0 >> 13) & 0xFFu), w1, astar, true, sbest, kbest);
                    if (++cq == nca) { cq = 0; uq++; }
                }
            }
        }
        unsigned long long mkey = ~0ull;
        if constexpr (PRUNE) {
            // Moves off the critical client, with their ids (a move that wins is then known without a second
            // look): every wave takes every segment of the client and a slice of the target clients, which
            // keeps all waves busy where clients are many and small.
            const int mb = min(max(uni(l.gstart[astar]), 0), P), me = min(max(uni(l.gstart[astar + 1]), mb), P);
            if (nfeas > 0)
                for (int p0 = mb; p0 < me; p0 += kWave) {                    // (the client's range may end inside a segment)
                    const bool in = p0 + lane < me;
                    const uint32_t x = in ? l.cu[p0 + lane] : kPad, jb = in ? (uint32_t)l.job[p0 + lane] : 0u;
                    if (wave == 0) w_cnt += (uint32_t)__popcll(__ballot(x != kPad)) * (uint32_t)(M - 1);
                    const uint32_t ci = (x - kBias) >> 1;
                    const uint32_t la = load32(astar);
                    uint32_t bv = kInf, bid = kInf;
                    for (int q = wave; q < nfeas; q += kWaves) {
                        const int b = l.feas[q];
                        if (b == astar) continue;
                        const uint32_t v = max(max(la - ci, load32(b) + ci), others_max(top, astar, b));
                        const uint32_t id = jb * (uint32_t)M + (uint32_t)b;
                        const bool better = v < bv || (v == bv && id < bid);
                        bv = better ? v : bv;
                        bid = better ? id : bid;
                    }
                    if (x != kPad && bv != kInf) mkey = min(mkey, ((unsigned long long)bv << 32) | (unsigned long long)bid);
                }
            if (nfeas > 0) {
                mkey = wave_min_u64(mkey);
                mbest = (uint32_t)(mkey >> 32);              // (kInf when this wave saw no move)
            }
        } else {
            if (nfeas > 0) mbest = wave_min_u32(mbest);
        }
        sbest = wave_min_u32(sbest);
        kbest = wave_min_u64(kbest);
        if (lane == 0) {
            if (mbest != kInf) {
                atomicMin(&ctrl->vmove, mbest);
                if constexpr (PRUNE) atomicMin(&ctrl->kmove, mkey);
            }
            if (sbest != kInf) atomicMin(&ctrl->vswap, sbest);
            if (kbest != ~0ull) atomicMin(&ctrl->k0key, kbest);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");       // this wave's minima (rowkey included) before its post
        if (lane == 0) atomicAdd(&ctrl->adone, 1);

        // ---- phase B (wave 0): which candidate; nothing is changed before B2.  Only wave 0 needs
        //      the values of phase A: it waits for the other waves' contributions on a counter (they
        //      never wait for wave 0 before they post it) while they go straight on to phase C. ----
        int act = kActNone;
        unsigned long long win = ~0ull;
        uint32_t Vm = kInf, Vs = kInf, V = kInf;
        if (wave == 0) {
            int posted = 0;
            for (int spins = 0; spins < kSpinLimit; spins++) {
                if (lane == 0) posted = atomicAdd(&ctrl->adone, 0);
                posted = uni(posted);
                if (posted >= kWaves) break;
                __builtin_amdgcn_s_sleep(1);
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
            Vm = uniu(ctrl->vmove); Vs = uniu(ctrl->vswap);
            V = min(Vm, Vs);
            if (posted < kWaves) act = kActError;        // cannot happen: a wave never posted
        }
        if (wave == 0) {
            if (act == kActError) { }
            else if (V >= T) act = kActStop;                  // local optimum (status stays OK)
            else if (Vm <= Vs) {
                unsigned long long best = ~0ull;
                if constexpr (PRUNE) {
                    // ---- a move wins (move ids are below swap ids): phase A left the lowest id among the moves of
                    //      value V; its job sits in one of the critical client's segments ----
                    const unsigned long long km = ctrl->kmove;
                    const uint32_t id = uniu((uint32_t)km);
                    const uint32_t ji = id / (uint32_t)M;
                    const int mb = min(max(uni(l.gstart[astar]), 0), P), me = min(max(uni(l.gstart[astar + 1]), mb), P);
                    if ((uint32_t)(km >> 32) == V)
                        for (int p0 = mb; p0 < me; p0 += kWave) {
                            const int p = p0 + lane;
                            if (p < me && l.cu[p] != kPad && (uint32_t)l.job[p] == ji) best = ((unsigned long long)id << 32) | (unsigned long long)p;
                        }
                } else {
                    // ---- a move wins (move ids are below swap ids): lowest id among moves of value V.  V is
                    //      below the makespan, so the job leaves the critical client: only its segments are scanned ----
                    for (int seg = sega; seg < segb; seg++) {
                        const int g = astar;
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
                }
                win = wave_min_u64(best);
                act = kActMove;
            } else {
                // ---- a swap wins: lowest (min(i,k), max(i,k)) among swaps of value V.  Its other job f is
                // flagged (rowkey[f] == V).  k0 = the lowest-index flagged job.  Candidates: k0 with its
                // critical partners, and the critical jobs with a lower index than k0 ("early") with theirs. ----
                const unsigned long long k0key = ctrl->k0key;
                if ((uint32_t)(k0key >> 32) != V) act = kActError;      // cannot happen: the best swap is in a critical tile
                else {
                    const uint32_t k0job = uniu((uint32_t)(k0key >> 16) & 0xFFFFu);
                    const int k0pos = min(uni((int)(k0key & 0xFFFFu)), P - 1);
                    const uint32_t lstar = wload(astar);
                    const int sbase = min(max(uni(l.gstart[astar]), 0), P), scnt = min(max(uni(l.cnt[astar]), 0), P - sbase);
                    const int send = sbase + scnt;
                    unsigned long long best = ~0ull;

                    // all critical jobs against the flagged job at pf (uniform): every swap of value V
                    auto pair_with = [&](int pf) {
                        const int g = uni(l.seg_grp[pf >> kGrpShift]);
                        const uint32_t lg = wload(g), jf = uniu(l.job[pf]);
                        const uint32_t xf = uniu(l.cu[pf]) - (lg - lstar);
                        const uint32_t oth = others_max(top, g, astar);
                        for (int p = sbase + lane; p < send; p += kWave) {
                            const uint32_t je = l.job[p];
                            if (swap_value(absdiff_u32(l.cu[p], xf), lg + lstar, oth) == V) {
                                const unsigned long long lo = je < jf ? ((unsigned long long)je << 48) | ((unsigned long long)jf << 32) |
                                                                            ((unsigned long long)p << 16) | (unsigned long long)pf
                                                                      : ((unsigned long long)jf << 48) | ((unsigned long long)je << 32) |
                                                                            ((unsigned long long)pf << 16) | (unsigned long long)p;
                                best = min(best, lo);
                            }
                        }
                    };
                    pair_with(k0pos);

                    // early critical jobs: are there any?
                    int nE = 0;
                    for (int p0 = sbase; p0 < send; p0 += kWave) {
                        const int p = p0 + lane;
                        nE += __popcll(__ballot(p < send && (uint32_t)l.job[p] < k0job));
                    }
                    if (nE > 0) {
                        // Per client g, for a flagged job f of g and a critical job e: the swap has value V
                        // <=> |cu_e - (cu_f - tdl[g])| < tr1[g]  (tr1 = 0: no swap with g reaches V).
                        for (int g = lane; g < M; g += kWave) {
                            const uint32_t lg = load32(g), lsum = lg + lstar;
                            const bool ok = g != astar && others_max(top, g, astar) <= V && lsum <= 2u * V + 1u;
                            l.tdl[g] = lg - lstar;
                            l.tr1[g] = ok ? 2u * V + 2u - lsum : 0u;
                        }
                        __builtin_amdgcn_wave_barrier();
                        const uint4 *cu4 = reinterpret_cast<const uint4 *>(l.cu);
                        const uint4 *rk4 = reinterpret_cast<const uint4 *>(l.rowkey);
                        const uint2 *rk2 = reinterpret_cast<const uint2 *>(l.rowkey16);
                        const uint2 *job2 = reinterpret_cast<const uint2 *>(l.job);
                        // The early jobs are taken in increasing index order, four at a time, each batch against
                        // every flagged job; the first batch with a partner holds the lowest id (a partner f of an
                        // early job e is flagged, so job(f) >= job(k0) > job(e)).  If the first batch finds nothing
                        // and few jobs are flagged, those are paired with all critical jobs instead.
                        int lastjob = -1, nF = 0, nrec = 0;
                        int f0 = 0, f1 = 0, f2 = 0, f3 = 0;
                        for (int round = 0; round * 4 < nE; round++) {
                            int ne = 0;
                            uint32_t ecu0 = 0, ecu1 = 0, ecu2 = 0, ecu3 = 0, ejp0 = 0, ejp1 = 0, ejp2 = 0, ejp3 = 0;   // cu, job << 16 | pos
                            for (int k = 0; k < 4; k++) {
                                uint32_t m = kInf;
                                for (int p = sbase + lane; p < send; p += kWave) {
                                    const uint32_t je = l.job[p];
                                    if ((int)je > lastjob && je < k0job) m = min(m, (je << 16) | (uint32_t)p);
                                }
                                m = wave_min_u32(m);
                                if (m == kInf) break;
                                lastjob = (int)(m >> 16);
                                ecu3 = ecu2; ecu2 = ecu1; ecu1 = ecu0;
                                ejp3 = ejp2; ejp2 = ejp1; ejp1 = ejp0;
                                ejp0 = m;
                                ecu0 = uniu(l.cu[min((int)(m & 0xFFFFu), P - 1)]);
                                ne += 1;
                            }
                            if (ne == 0) break;
                            uint32_t b0 = kInf, b1 = kInf, b2 = kInf, b3 = kInf;   // per early job: lowest (job << 16 | pos) partner
                            for (int q0 = 0; q0 < (P >> 2); q0 += kWave) {
                                const int q = q0 + lane;                            // positions 4q .. 4q+3 (P % 256 == 0 is not given)
                                const bool in = q < (P >> 2);
                                const int g = in ? min((int)l.seg_grp[q >> (kGrpShift - 2)], M - 1) : 0;
                                const uint4 cc = in ? cu4[q] : make_uint4(kPad, kPad, kPad, kPad);
                                uint4 rr = make_uint4(kInf, kInf, kInf, kInf);
                                if constexpr (PRUNE) {
                                    // 16 bits per row: a row whose low bits match is re-checked by the key test below
                                    // (a candidate of value V passes it, nothing else does), so a chance match costs
                                    // nothing but its place in the count of flagged rows
                                    if (in) {
                                        const uint2 r2 = rk2[q];
                                        const uint32_t hiV = V & 0xFFFF0000u;
                                        rr = make_uint4(hiV | (r2.x & 0xFFFFu), hiV | (r2.x >> 16), hiV | (r2.y & 0xFFFFu), hiV | (r2.y >> 16));
                                    }
                                } else if (in) rr = rk4[q];
                                const uint2 jj = in ? job2[q] : uint2{0u, 0u};
                                const uint32_t dl = l.tdl[g], r1 = l.tr1[g];
                                const uint32_t pq = (uint32_t)q << 2;
                                const uint32_t x[4] = {cc.x - dl, cc.y - dl, cc.z - dl, cc.w - dl};
                                const bool fl[4] = {rr.x == V, rr.y == V, rr.z == V, rr.w == V};
                                const uint32_t id[4] = {fl[0] ? ((jj.x & 0xFFFFu) << 16) | pq : kInf,
                                                        fl[1] ? (jj.x & 0xFFFF0000u) | (pq + 1u) : kInf,
                                                        fl[2] ? ((jj.y & 0xFFFFu) << 16) | (pq + 2u) : kInf,
                                                        fl[3] ? (jj.y & 0xFFFF0000u) | (pq + 3u) : kInf};
#pragma unroll
                                for (int k = 0; k < 4; k++) {
                                    if (round == 0) {                               // count the flagged jobs, keep the first four
                                        unsigned long long m = __ballot(fl[k]);
                                        nF += __popcll(m);
                                        while (m && nrec < 4) {
                                            const int ln = __builtin_ctzll(m);
                                            m &= m - 1;
                                            f3 = f2; f2 = f1; f1 = f0;
                                            f0 = ((q0 + ln) << 2) + k;
                                            nrec += 1;
                                        }
                                    }
                                    b0 = min(b0, absdiff_u32(ecu0, x[k]) < r1 ? id[k] : kInf);
                                    if (ne > 1) b1 = min(b1, absdiff_u32(ecu1, x[k]) < r1 ? id[k] : kInf);
                                    if (ne > 2) b2 = min(b2, absdiff_u32(ecu2, x[k]) < r1 ? id[k] : kInf);
                                    if (ne > 3) b3 = min(b3, absdiff_u32(ecu3, x[k]) < r1 ? id[k] : kInf);
                                }
                            }
                            auto early_pair = [&](uint32_t ejp, uint32_t b) {
                                if (b != kInf)
                                    best = min(best, ((unsigned long long)(ejp >> 16) << 48) | ((unsigned long long)(b >> 16) << 32) |
                                                         ((unsigned long long)(ejp & 0xFFFFu) << 16) | (unsigned long long)(b & 0xFFFFu));
                            };
                            early_pair(ejp0, b0);
                            if (ne > 1) early_pair(ejp1, b1);
                            if (ne > 2) early_pair(ejp2, b2);
                            if (ne > 3) early_pair(ejp3, b3);
                            if (__ballot(min(min(b0, b1), min(b2, b3)) != kInf)) break;
                            if (round == 0 && nF <= 4) {
                                if (nrec > 0 && f0 != k0pos) pair_with(min(f0, P - 1));
                                if (nrec > 1 && f1 != k0pos) pair_with(min(f1, P - 1));
                                if (nrec > 2 && f2 != k0pos) pair_with(min(f2, P - 1));
                                if (nrec > 3 && f3 != k0pos) pair_with(min(f3, P - 1));
                                break;
                            }
                        }
                    }
                    win = wave_min_u64(best);
                    act = kActSwap;
                }
            }
        }

        // what the apply step will need, read while nothing has changed (wave 0)
        int ap_g0 = 0, ap_g1 = 0, ap_j0 = 0, ap_j1 = 0;
        uint32_t ap_x0 = 0, ap_x1 = 0;
        if (act == kActMove) {
            const uint32_t id = (uint32_t)(win >> 32);
            const int p = (int)(uint32_t)win;
            ap_j0 = (int)(id / (uint32_t)M); ap_g1 = (int)(id % (uint32_t)M);
            if (win == ~0ull || ap_j0 >= N || p >= P) act = kActError;       // cannot happen: the best move was found above
            else { ap_g0 = uni(l.seg_grp[p >> kGrpShift]); ap_x0 = (uniu(l.cu[p]) - kBias) >> 1; }
        } else if (act == kActSwap) {
            ap_j0 = (int)(uint32_t)(win >> 48); ap_j1 = (int)((uint32_t)(win >> 32) & 0xFFFFu);                  // j0 < j1
            const int pi = (int)((win >> 16) & 0xFFFFu), pk = (int)(win & 0xFFFFu);
            if (win == ~0ull || ap_j0 >= N || ap_j1 >= N || pi >= P || pk >= P) act = kActError;               // cannot happen
            else {
                ap_g0 = uni(l.seg_grp[pi >> kGrpShift]); ap_g1 = uni(l.seg_grp[pk >> kGrpShift]);
                ap_x0 = uniu(l.cu[pi]); ap_x1 = uniu(l.cu[pk]);
            }
        }

        // ---- phase C: the rest of the scan, dealt from a counter: the swap tiles of the task table
        //      that do not involve the critical client, then the move segments of the other clients ----
        if constexpr (!PRUNE) {
            uint32_t rbest = kInf;
            unsigned long long knone = ~0ull;
            const int nwork = ntask + (nfeas > 0 ? nseg : 0);
            for (;;) {
                int t = 0;
                if (lane == 0) t = atomicAdd(&ctrl->next, 1);
                t = uni(t);
                if (t >= nwork || t < 0) break;
                const unsigned long long rec = t < ntask ? l.tasks[t] : 0ull;
                if (t < ntask) {
                    const uint32_t w0 = uniu((uint32_t)rec), w1 = uniu((uint32_t)(rec >> 32));
                    const int X = (int)((w0 >> 13) & 0xFFu), Y = (int)((w1 >> 19) & 0xFFu);
                    if (X != astar && Y != astar) run(w0, X, w1, Y, false, rbest, knone);
                } else {
                    const int seg = t - ntask;
                    const int g = l.seg_grp[seg];
                    if (g != astar) rbest = min(rbest, segment_moves(seg, g));
                }
            }
            rbest = wave_min_u32(rbest);
            if (lane == 0 && rbest != kInf) atomicMin(&ctrl->vrest, rbest);
            if (lane == 0 && w_cnt != 0) atomicAdd(&ctrl->counted, w_cnt);
        }
        __syncthreads();                                 // B2: the scan is complete
        if (wave != 0) {                                 // the waves that now wait put the row minima back to "none"
            uint4 *rk = reinterpret_cast<uint4 *>(l.rowkey);
            for (int q = tid - kWave; q < (P >> (PRUNE ? 3 : 2)); q += BLOCK - kWave) rk[q] = make_uint4(kInf, kInf, kInf, kInf);
            continue;
        }

        // ---- wave 0: apply (its operands were read before the barrier), open the next pass ----
        uint32_t vnew = vload;
        if (!PRUNE && uniu(ctrl->vrest) < T) act = kActError;       // cannot happen: those candidates keep the critical load
        {
            // The candidates of the scan: N (M - 1) moves and every pair on different clients.  The full
            // scan reports what its waves counted while they ran the tiles and the move segments (moves
            // whose targets are all full are the uniform capacity test: counted here) and stops the
            // scenario if that is not the whole neighbourhood; the pruned scan reports the same number,
            // which is by definition what a full scan would have enumerated.
            const unsigned long long whole = (unsigned long long)N * (unsigned long long)(M - 1) + w_pairs;
            if constexpr (PRUNE) w_evals += whole;
            else {
                unsigned long long counted = (unsigned long long)ctrl->counted;
                if (nfeas == 0) counted += (unsigned long long)N * (unsigned long long)(M - 1);
                if (counted != whole) act = kActError;
                w_evals += counted;
            }
        }
        if (act == kActStop) {
            if (lane == 0) ctrl->stop = 1;
            continue;
        }
        if (act == kActMove) {
            const uint32_t ci = ap_x0;
            const int a = ap_g0, b = ap_g1, i = ap_j0;
            if (SMALLM) {
                vnew = vload - (lane == a ? ci : 0u) + (lane == b ? ci : 0u);
                if (lane == a || lane == b) l.load[lane] = (long long)vnew;
            }
            bool in_place = false;
            if constexpr (PRUNE) {
                // Sorted layout, no tile tables: the job leaves its client's range (the later entries move down)
                // and enters the target's at its place (the later entries move up) when the target's range has
                // a free position; only a full range needs the jobs regrouped.
                const int p = (int)(uint32_t)win;
                const int ga0 = min(max(uni(l.gstart[a]), 0), P), na = min(max(uni(l.cnt[a]), 0), P - ga0);
                const int gb0 = min(max(uni(l.gstart[b]), 0), P), gb1 = min(max(uni(l.gstart[b + 1]), 0), P);
                const int nb = min(max(uni(l.cnt[b]), 0), P - gb0);
                if (gb0 + nb < gb1 && p >= ga0 && p < ga0 + na) {
                    in_place = true;
                    const uint32_t x = 2u * ci + kBias;
                    const int last = ga0 + na - 1;
                    for (int p0 = p; p0 < last; p0 += kWave) {             // entries (p, last] move down by one
                        const int q = p0 + lane;
                        const bool in = q < last;
                        const uint32_t v = in ? l.cu[q + 1] : 0u;
                        const uint16_t jv = in ? l.job[q + 1] : (uint16_t)0;
                        __builtin_amdgcn_wave_barrier();
                        if (in) { l.cu[q] = v; l.job[q] = jv; }
                        __builtin_amdgcn_wave_barrier();
                    }
                    if (lane == 0) { l.cu[last] = kPad; l.job[last] = kNoJob; }
                    int less = 0;
                    for (int p0 = gb0; p0 < gb0 + nb; p0 += kWave) {
                        const int q = p0 + lane;
                        less += __popcll(__ballot(q < gb0 + nb && l.cu[q] < x));
                    }
                    const int t = gb0 + less;
                    for (int p1 = gb0 + nb; p1 > t; p1 -= kWave) {         // entries [t, end) move up by one
                        const int q = p1 - lane;
                        const bool in = q > t;
                        const uint32_t v = in ? l.cu[q - 1] : 0u;
                        const uint16_t jv = in ? l.job[q - 1] : (uint16_t)0;
                        __builtin_amdgcn_wave_barrier();
                        if (in) { l.cu[q] = v; l.job[q] = jv; }
                        __builtin_amdgcn_wave_barrier();
                    }
                    if (lane == 0) { l.cu[t] = x; l.job[t] = (uint16_t)i; }
                    // pairs on different clients: (N^2 - sum n^2) / 2 falls by n_b - n_a + 1
                    w_pairs = (unsigned long long)((long long)w_pairs - ((long long)nb - (long long)na + 1));
                }
            }
            if (lane == 0) {
                if (!SMALLM) { l.load[a] -= (long long)ci; l.load[b] += (long long)ci; }
                l.cnt[a] -= 1; l.cnt[b] += 1;
                asg[i] = b;
                if (applied_log) applied_log[(size_t)s * max_passes + w_passes] = (uint64_t)(uint32_t)(win >> 32);
                if (in_place) ctrl->pairs_per_scan = w_pairs;
                else ctrl->rebuild = 1;
            }
            if (in_place) {                                  // move targets: the clients below the limit, ascending
                __builtin_amdgcn_wave_barrier();
                int nf = 0;
                for (int j0 = 0; j0 < M; j0 += kWave) {
                    const int j = j0 + lane;
                    const bool ok = j < M && l.cnt[j] < cap;
                    const unsigned long long m = __ballot(ok);
                    if (ok) l.feas[nf + __popcll(m & ((1ull << lane) - 1ull))] = j;
                    nf += __popcll(m);
                }
                if (lane == 0) ctrl->nfeas = nf;
            }
            w_passes += 1;
        } else if (act == kActSwap) {
            const int ga = ap_g0, gb = ap_g1;
            const uint32_t xi = ap_x0, xk = ap_x1;
            const uint32_t ji = (uint32_t)ap_j0, jk = (uint32_t)ap_j1;
            const int pi = (int)((win >> 16) & 0xFFFFu), pk = (int)(win & 0xFFFFu);
            const uint32_t d = ((xi - kBias) >> 1) - ((xk - kBias) >> 1);     // modulo 2^32; the loads stay in range
            if (SMALLM) {
                vnew = vload - (lane == ga ? d : 0u) + (lane == gb ? d : 0u);
                if (lane == ga || lane == gb) l.load[lane] = (long long)vnew;
            }
            if constexpr (PRUNE) {
                // the clients' positions stay sorted: the entry at pr leaves, (xnew, jnew) enters where it belongs
                auto replace_sorted = [&](int g, int pr, uint32_t xnew, uint32_t jnew) {
                    const int gb0 = min(max(uni(l.gstart[g]), 0), P), n = min(max(uni(l.cnt[g]), 0), P - gb0);
                    if (pr < gb0 || pr >= gb0 + n) return;              // cannot happen: the entry is one of the client's
                    int less = 0;
                    for (int p0 = gb0; p0 < gb0 + n; p0 += kWave) {
                        const int p = p0 + lane;
                        less += __popcll(__ballot(p < gb0 + n && p != pr && l.cu[p] < xnew));
                    }
                    const int t = gb0 + less;                          // where the new entry goes
                    if (t > pr) {
                        for (int p0 = pr; p0 < t; p0 += kWave) {       // entries (pr, t] move down by one
                            const int p = p0 + lane;
                            const bool in = p < t;
                            const uint32_t v = in ? l.cu[p + 1] : 0u;
                            const uint16_t jv = in ? l.job[p + 1] : (uint16_t)0;
                            __builtin_amdgcn_wave_barrier();
                            if (in) { l.cu[p] = v; l.job[p] = jv; }
                            __builtin_amdgcn_wave_barrier();
                        }
                    } else if (t < pr) {
                        for (int p1 = pr; p1 > t; p1 -= kWave) {       // entries [t, pr) move up by one
                            const int p = p1 - lane;
                            const bool in = p > t;
                            const uint32_t v = in ? l.cu[p - 1] : 0u;
                            const uint16_t jv = in ? l.job[p - 1] : (uint16_t)0;
                            __builtin_amdgcn_wave_barrier();
                            if (in) { l.cu[p] = v; l.job[p] = jv; }
                            __builtin_amdgcn_wave_barrier();
                        }
                    }
                    if (lane == 0) { l.cu[t] = xnew; l.job[t] = (uint16_t)jnew; }
                };
                replace_sorted(ga, pi, xk, jk);
                replace_sorted(gb, pk, xi, ji);
            }
            if (lane == 0) {
                if (!SMALLM) { l.load[ga] -= (long long)(int32_t)d; l.load[gb] += (long long)(int32_t)d; }
                if constexpr (!PRUNE) {
                    l.cu[pi] = xk; l.cu[pk] = xi;
                    l.job[pi] = (uint16_t)jk; l.job[pk] = (uint16_t)ji;
                }
                asg[ji] = gb; asg[jk] = ga;
                if (applied_log)
                    applied_log[(size_t)s * max_passes + w_passes] =
                        (uint64_t)N * (uint64_t)M + (uint64_t)ji * (uint64_t)N + (uint64_t)jk;
            }
            w_passes += 1;
        }
        if (act == kActError || act == kActNone) { w_status = MMBP_ST_INTERNAL; w_stop = true; }
        open_pass(vnew, false);
    }

    // ---------------- write back ----------------
    __syncthreads();
    for (int j = tid; j < M; j += BLOCK) load_out[(size_t)s * M + j] = l.load[j];
    if (tid == 0) {
        long long t = 0;
        for (int j = 0; j < M; j++) t = max(t, l.load[j]);
        makespan_out[s] = t;
        passes_out[s] = w_passes;
        if (evals_out) evals_out[s] = w_evals;
        status_out[s] = w_status;
    }
}

template <typename CostT, int BLOCK, bool SMALLM, bool PRUNE>
hipError_t launch_one(const void *cost, int S, int N, int M, int cap, int max_passes, int32_t *assign,
                      int64_t *load_out, int64_t *makespan_out, int32_t *passes_out, uint64_t *evals_out,
                      uint64_t *applied_log, int32_t *status_out, hipStream_t st)
{
    const size_t bytes = lds_bytes(N, M, PRUNE);
    if (bytes > 64 * 1024) {                             // beyond the default limit: raise it for this kernel (per device,
                                                         // cheap, so done at every such launch)
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&ls_lds_kernel<CostT, BLOCK, SMALLM, PRUNE>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit);
        if (e != hipSuccess) return e;
    }
    ls_lds_kernel<CostT, BLOCK, SMALLM, PRUNE><<<dim3(S), dim3(BLOCK), bytes, st>>>(
        (const CostT *)cost, N, M, cap, max_passes, assign, load_out, makespan_out, passes_out, evals_out,
        applied_log, status_out);
    return hipGetLastError();
}

}  // namespace

bool ls_lds_fits(int N, int M, bool prune)
{
    return N < 65535 && N + 64 * M <= 65536 && lds_bytes(N, M, prune) <= kLdsLimit;
}

hipError_t launch_ls_lds(const void *cost, int dtype, int S, int N, int M, int cap, int max_passes, int prune,
                         int32_t *assign, int64_t *load_out, int64_t *makespan_out, int32_t *passes_out,
                         uint64_t *evals_out, uint64_t *applied_log, int32_t *status_out, hipStream_t st)
{
    // workgroup size by padded problem size (1024 threads were measured slower at every size: a scan has
    // too few tiles for 16 waves)
    const int pmax = N + 64 * M;
    const int block = pmax <= 512 ? 256 : 512;
#define MMBP_LDS_LAUNCH(T, B, SM) \
    (prune ? launch_one<T, B, SM, true>(cost, S, N, M, cap, max_passes, assign, load_out, makespan_out, passes_out, evals_out, \
                                        applied_log, status_out, st) \
           : launch_one<T, B, SM, false>(cost, S, N, M, cap, max_passes, assign, load_out, makespan_out, passes_out, evals_out, \
                                         applied_log, status_out, st))
#define MMBP_LDS_PICK(T) \
    (block == 256 ? (M <= 64 ? MMBP_LDS_LAUNCH(T, 256, true) : MMBP_LDS_LAUNCH(T, 256, false)) \
                  : (M <= 64 ? MMBP_LDS_LAUNCH(T, 512, true) : MMBP_LDS_LAUNCH(T, 512, false)))
    if (dtype == MMBP_I32) return MMBP_LDS_PICK(int32_t);
    return MMBP_LDS_PICK(int64_t);
#undef MMBP_LDS_PICK
#undef MMBP_LDS_LAUNCH
}

}  // namespace mmbp
